/*
 * psf.h -- C ABI of libpsf: causal polynomial-sketch attention on AMD CDNA4 (gfx950).
 *
 * Entry points: psf_sketch, psf_causal_attn_fwd (the hot path), psf_noncausal_attn_fwd,
 * psf_causal_attn_bwd, psf_causal_attn_fwd_save + psf_causal_attn_bwd_saved (forward and
 * backward without a second forward pass), psf_decode_step (token by token) with
 * psf_decode_prefill (its state after a prompt), the *_timed variants for benchmarking, and the
 * host-only sizing / selection queries.
 *
 * Method: PolySketchFormer (arXiv 2310.01655).  Every query/key row x is mapped to
 *   m(x)    = PolySketchWithNegativity(x, r, p/2)            (Algorithm 1)
 *   phi'(x) = m(x) (x) m(x)  in R^{r^2}, index a*r + b       (Algorithm 1, PolySketchNonNegative)
 * and the causal, normalised attention of Section 3
 *   o_i = sum_{j<=i} w_ij v_j / (1 + sum_{j<=i} w_ij),   w_ij = <phi'(q_i), phi'(k_j)>
 * is evaluated with the block lower-triangular algorithm of Section 3.1 (per-block states
 * H_l = phi'(K_l)^T [V_l | 1], exclusive prefix Z_l over blocks, in-block term P_l) and, by
 * default, exact weights <q_i,k_j>^p for pairs inside one block (Section 3.2).  With
 * desc.learned the sketch m(x) is Algorithm 2's (small networks instead of Gaussian matrices).
 *
 * Conventions
 *   - Every data pointer is DEVICE memory owned by the caller.  The library never allocates,
 *     frees or synchronises; all work is enqueued on `hip_stream` (a hipStream_t, NULL = the
 *     default stream).  Calls are re-entrant as long as workspaces do not overlap.
 *   - Tensors are dense row-major: Q, K, M [batch, heads, n, d|r]; V, O [batch, heads, n, dv].
 *   - The library neither normalises Q/K (the paper applies layer normalisation before the
 *     kernel, Section 2.1) nor applies a 1/sqrt(d) scale (the final definition has none).
 *   - Sketch matrices G are data, not drawn here: [sets, g_len] with sets = heads when
 *     sketch_per_head != 0, else 1 (the paper shares one phi' per layer, Section 4), and inside
 *     a set the p/2 matrices of shape d x r followed by the p/2 - 2 matrices of shape r x r
 *     (counts: Theorem 1.1 item 3), each list in the order Algorithm 1 reaches its sampling
 *     line (left subtree, right subtree, node).  For p = 8: G1,G2 -> M1; G3,G4 -> M2; then the
 *     r x r pair applied to M1 and M2.  Same storage dtype as Q.
 *   - Errors are reported by return code only; arguments are validated on the host before
 *     anything is launched.  On error the contents of outputs and workspace are unspecified.
 */
#ifndef PSF_H
#define PSF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PSF_OK = 0,
    PSF_ERR_NULL = 1,        /* a required pointer is NULL                                  */
    PSF_ERR_SHAPE = 2,       /* non-positive size, or n not a multiple of b                 */
    PSF_ERR_UNSUPPORTED = 3, /* p not in {2,4,8,16}, feature count above PSF_MAX_FEATURES,
                                unknown enum value, sizes beyond the stated limits          */
    PSF_ERR_WORKSPACE = 4,   /* workspace smaller than psf_workspace_bytes()                */
    PSF_ERR_HIP = 5,         /* a HIP call or kernel launch failed                          */
    PSF_ERR_ALIGNMENT = 6    /* a tensor is not 16-byte aligned where the bf16 MFMA kernels,
                                which move 16-byte pieces, would run (psf_kernel_path == 1)  */
} psf_status;

typedef enum { PSF_F32 = 0, PSF_BF16 = 1 } psf_dtype;   /* storage type of Q, K, V, G, M, Phi, O */
typedef enum { PSF_FEAT_SKETCH = 0,                     /* phi' of Algorithm 1                   */
               PSF_FEAT_EXACT = 1 } psf_feat;           /* phi(x) = x^{(x)p} (Section 2.2), needs
                                                           d^p <= PSF_MAX_FEATURES               */
typedef enum { PSF_LOCAL_EXACT = 0,                     /* in-block weights <q,k>^p (Section 3.2) */
               PSF_LOCAL_SKETCH = 1 } psf_local;        /* in-block weights <phi',phi'> = <m,m>^2
                                                           (Section 3.1, the (L R^T)^2 shortcut)  */

#define PSF_MAX_FEATURES 65536   /* largest explicit feature count (r^2, d^2 for p = 2, or d^p) */
#define PSF_MAX_DIM 256          /* largest d, dv and r                                         */

/* Problem descriptor (plain data, passed by pointer, read on the host only). */
typedef struct {
    int32_t batch, heads;    /* units = batch * heads independent attention problems           */
    int32_t n;               /* context length                                                 */
    int32_t d, dv;           /* row length of Q/K and of V/O                                   */
    int32_t p;               /* polynomial degree: 2, 4, 8 or 16 (Algorithm 1 halves it)       */
    int32_t r;               /* sketch size; r^2 features.  Ignored for p = 2 and FEAT_EXACT   */
    int32_t b;               /* block size of the lower-triangular algorithm; n % b == 0       */
    int32_t dtype;           /* psf_dtype                                                      */
    int32_t feat;            /* psf_feat                                                       */
    int32_t local;           /* psf_local (ignored with FEAT_EXACT: all weights are exact)     */
    int32_t sketch_per_head; /* 0: one set of G for all heads, 1: G has a leading [heads] axis */
    int32_t learned;         /* 0: Gaussian sketch matrices (Algorithm 1); 1: learned sketches
                                (Algorithm 2, Appendix D): G then holds the networks' parameters,
                                psf_learned_len(d, r, p) entries per set.  p in {2, 4, 8}         */
} psf_desc;

/* Host-only check of a descriptor; what the other entry points run first. */
psf_status psf_check_desc(const psf_desc *desc);

/* Which kernels the descriptor selects: 1 = bf16 MFMA path (FEAT_SKETCH, bf16, p in {4,8},
 * r in {32,64}, d = dv in {64,128}, b % 256 == 0; LOCAL_EXACT, or LOCAL_SKETCH with Gaussian
 * sketches unless d = 128 and r = 32; also p = 2 with d = dv = 64, where m(x) = x and r is
 * ignored), 0 = general fp32 path
 * (everything else the descriptor check admits), -1 = invalid descriptor. */
int psf_kernel_path(const psf_desc *desc);

/* Which work psf_causal_attn_fwd runs inside the launch of its state kernel (the stage that
 * psf_stage_name(1, 2) calls "block_states_scan"), for a benchmark that splits flops by stage:
 * bit 0: the in-block part of the output (Section 3.2; the "output" stage is then the
 * cross-block part and the division only) and the scan of the denominator partials; bit 1: the
 * sketch of the query rows (Algorithm 1).  0 where none of this applies.  Host only. */
int psf_fwd_beside_states(const psf_desc *desc);

/* Bytes of device workspace psf_causal_attn_fwd needs for this descriptor (0 if invalid).
 * Holds the sketches m(Q), m(K), the block prefix states Z_l (Section 3.1) and staging. */
size_t psf_workspace_bytes(const psf_desc *desc);

/* Number of entries of one set of sketch matrices for (d, r, p). */
size_t psf_g_len(int32_t d, int32_t r, int32_t p);

/*
 * Learned sketches (Algorithm 2, Appendix D): every projection M G of Algorithm 1 is replaced by
 * a dense network f(M) and the Hadamard product is wrapped as sqrt(r) tanh(sqrt(1/r) f1 * f2).
 * Reading of the appendix taken here: f(a) = gelu(gelu(LN(a) W1) -> LN -> W2 -> W3) W4 with
 * hidden sizes 8r, r, 8r, output r, no dense biases (the appendix counts 8 h r + 24 r^2
 * parameters per network), layer normalisation (scale, bias, eps 1e-6, biased variance) before
 * the input and before the second hidden layer, gelu in its tanh form.  One set of parameters
 * is the p - 2 networks in the order the recursion reaches them (left subtree, right subtree,
 * then f1, f2 of the node), each stored as [g1, b1, W1 (in x 8r), g2, b2, W2 (8r x r),
 * W3 (r x 8r), W4 (8r x r)], matrices row-major with the input index first, in desc->dtype.
 * psf_learned_len returns the entries of one set (0 for p = 2).
 */
size_t psf_learned_len(int32_t d, int32_t r, int32_t p);

/*
 * psf_sketch -- Algorithm 1 applied to every row of X [batch, heads, n, d] (device).
 *   M_out   [batch, heads, n, r]    m(x) = PolySketchWithNegativity(x, r, p/2); r -> d when p = 2
 *   Phi_out [batch, heads, n, r*r]  phi'(x) = m(x) (x) m(x), or NULL to skip it.  With
 *                                   FEAT_EXACT: [.., n, d^p] = x^{(x)p} and M_out may be NULL.
 * G as described above (device; may be NULL when p = 2 or FEAT_EXACT).  Outputs are written
 * once, in desc->dtype (bf16 rounds to nearest even).  At least one output must be given.
 */
psf_status psf_sketch(const psf_desc *desc, const void *X, const void *G,
                      void *M_out, void *Phi_out, void *hip_stream);

/*
 * psf_causal_attn_fwd -- Section 3 causal Polysketch attention through the block algorithm of
 * Sections 3.1/3.2 with block size desc->b.
 *   Q, K [batch, heads, n, d], V [batch, heads, n, dv], G: device inputs (never written)
 *   O    [batch, heads, n, dv]: device output in desc->dtype
 *   workspace: device scratch of at least psf_workspace_bytes(desc) bytes, 256-byte aligned;
 *              contents on entry are irrelevant, contents on return unspecified.
 * Where psf_kernel_path(desc) == 1 the tensors must be 16-byte aligned (PSF_ERR_ALIGNMENT
 * otherwise; the same holds for the non-causal, backward, saved-state and prompt entry points
 * when they run the bf16 MFMA kernels).  Accumulation is fp32 throughout; on the MFMA path the operands of the contractions
 * (m(x), phi', Z_l, in-block weights) are rounded to bf16.
 */
psf_status psf_causal_attn_fwd(const psf_desc *desc, const void *Q, const void *K, const void *V,
                               const void *G, void *O,
                               void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * psf_causal_attn_fwd_static -- the same call for callers that cannot allocate device memory or
 * pass a workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The workspace is an array of PSF_STATIC_SCRATCH_BYTES bytes that lives in the
 * library's device image (one copy per GPU, held until the process ends); the call allocates and
 * frees nothing and runs the same kernels as psf_causal_attn_fwd, so the output is the same bit
 * for bit.  Inputs and output are still the caller's.
 *   Problems with psf_workspace_bytes(desc) > PSF_STATIC_SCRATCH_BYTES are rejected with
 *   PSF_ERR_WORKSPACE before anything is launched (use psf_causal_attn_fwd for those).
 *   All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU
 *   (different streams, or different host threads) race and give unspecified results;
 *   calls on one stream are ordered and safe.  Nothing in the array has to survive between
 *   calls and nothing needs clearing.  The first call on a device looks the array's address up
 *   (once per device, with that device current); later calls only enqueue kernels.
 */
#define PSF_STATIC_SCRATCH_BYTES (32u << 20)
psf_status psf_causal_attn_fwd_static(const psf_desc *desc, const void *Q, const void *K, const void *V,
                                      const void *G, void *O, void *hip_stream);

/*
 * Same call, but brackets each kernel with HIP events on `hip_stream`, waits for the stream
 * and reports per-stage milliseconds: stage_ms[i], stage names via psf_stage_name(path, i).
 * n_stages is the capacity of stage_ms; returns the stage count in *n_written.  Creates and
 * destroys HIP events; intended for benchmarking only.
 */
psf_status psf_causal_attn_fwd_timed(const psf_desc *desc, const void *Q, const void *K,
                                     const void *V, const void *G, void *O,
                                     void *workspace, size_t workspace_bytes, void *hip_stream,
                                     float *stage_ms, int32_t n_stages, int32_t *n_written);
const char *psf_stage_name(int path, int32_t stage);

/*
 * psf_noncausal_attn_fwd -- Polysketch attention without a mask (Section 2.2):
 *   O = D^-1 phi'(Q) phi'(K)^T V,  D = diag(1 + phi'(Q) phi'(K)^T 1)
 * i.e. o_i = sum over ALL j of w_ij v_j / (1 + sum_j w_ij), w_ij = <phi'(q_i), phi'(k_j)>
 * (PSF_FEAT_EXACT: w_ij = <q_i, k_j>^p).  Same descriptor, arguments, layouts, dtype rules and
 * error behaviour as psf_causal_attn_fwd; there is no in-block rule here, so `local` is ignored,
 * and `b` only partitions the work (it must still divide n).  Learned sketches are accepted.
 * The same two kernel paths (psf_kernel_path); the workspace size is its own:
 * psf_noncausal_workspace_bytes(desc).  One state per unit is built from all keys and applied
 * to every query: cost linear in n.  Stage names of the _timed variant: psf_stage_name(path, i)
 * of the causal call (the same kernels run).
 */
size_t psf_noncausal_workspace_bytes(const psf_desc *desc);
psf_status psf_noncausal_attn_fwd(const psf_desc *desc, const void *Q, const void *K, const void *V,
                                  const void *G, void *O,
                                  void *workspace, size_t workspace_bytes, void *hip_stream);
psf_status psf_noncausal_attn_fwd_timed(const psf_desc *desc, const void *Q, const void *K,
                                        const void *V, const void *G, void *O,
                                        void *workspace, size_t workspace_bytes, void *hip_stream,
                                        float *stage_ms, int32_t n_stages, int32_t *n_written);

/*
 * psf_causal_attn_bwd -- gradient of psf_causal_attn_fwd's output with respect to Q, K and V.
 * The paper trains through the attention of Section 3 (weights of Sections 3.1 / 3.2, sketch of
 * Algorithm 1); this is the chain rule through exactly that function, evaluated with the same
 * block decomposition: the prefix states Z_l of Section 3.1 for the query side and their mirror
 * image (sums over later blocks of phi'(q_i) [dO_i / D_i | -<dO_i, o_i> / D_i]^T) for keys and
 * values.  The sketch matrices G are constants (no gradient).
 *   Q, K, V, G as for the forward call; dO [batch, heads, n, dv]: dL/dO (device, never written)
 *   dQ, dK [batch, heads, n, d], dV [batch, heads, n, dv]: device outputs in desc->dtype,
 *   each written once; must not alias any input.
 *   workspace: at least psf_bwd_workspace_bytes(desc) bytes, 256-byte aligned.  The forward
 *   quantities are recomputed inside; nothing has to be kept from the forward call.
 * Supported: PSF_FEAT_SKETCH with either in-block rule, every p, r, d, dv, b and dtype the
 * descriptor check admits (fp32 arithmetic), Gaussian or learned sketches (with learned ones G
 * holds the networks' parameters and this call treats them as constants; see
 * psf_causal_attn_bwd_learned).  PSF_FEAT_EXACT returns PSF_ERR_UNSUPPORTED.
 * Kernels: bf16 storage with d = dv in {64, 128}, p in {4, 8}, r in {32, 64}, b % 256 == 0 and
 * PSF_LOCAL_EXACT (random sketches; learned ones for d = 64, p = 4) or PSF_LOCAL_SKETCH (random
 * sketches, d = r = 64, p = 4) runs on MFMA
 * (psf_bwd_kernel_path == 3; bf16 operands, fp32 accumulation, g and
 * the in-block weights rounded to bf16 like the forward pass rounds its weights; the learned
 * networks' layers take fp16 activations like the forward kernel, their gradients bf16);
 * everything else runs the general fp32 kernels (== 2).  -1: invalid descriptor or unsupported.
 * The _timed variant reports per-stage milliseconds like psf_causal_attn_fwd_timed, stage
 * names via psf_stage_name(psf_bwd_kernel_path(desc), i).
 */
int psf_bwd_kernel_path(const psf_desc *desc);
size_t psf_bwd_workspace_bytes(const psf_desc *desc);
psf_status psf_causal_attn_bwd(const psf_desc *desc, const void *Q, const void *K, const void *V,
                               const void *G, const void *dO, void *dQ, void *dK, void *dV,
                               void *workspace, size_t workspace_bytes, void *hip_stream);
psf_status psf_causal_attn_bwd_timed(const psf_desc *desc, const void *Q, const void *K,
                                     const void *V, const void *G, const void *dO, void *dQ,
                                     void *dK, void *dV, void *workspace, size_t workspace_bytes,
                                     void *hip_stream, float *stage_ms, int32_t n_stages,
                                     int32_t *n_written);

/*
 * psf_causal_attn_bwd_learned -- psf_causal_attn_bwd for desc->learned = 1 that also returns the
 * gradient with respect to the parameters of the learned sketch (Algorithm 2, Appendix D: the
 * networks are trained with the model, Section 2.3): the chain rule through
 * sqrt(r) tanh(f1(M1) * f2(M2) / sqrt(r)) at every node and through every network layer by
 * layer (dense layers, tanh-form gelu, layer normalisation), summed over the query and the key
 * rows that share a parameter set.
 *   dG [sets, psf_learned_len(d, r, p)] fp32 (device): overwritten, in G's parameter order;
 *   sets = heads when desc->sketch_per_head, else 1.  Everything else as for psf_causal_attn_bwd;
 *   workspace: psf_bwd_workspace_bytes(desc) (it includes the staging of the parameter sums).
 * The sums over rows run in a fixed order (no atomics: a repeated call returns the same bits).
 * Kernels as psf_bwd_kernel_path says: MFMA (== 3: the sums are then formed from bf16 operands,
 * fp32 accumulation) or the general fp32 ones (== 2).  PSF_ERR_UNSUPPORTED unless desc->learned
 * (and p > 2); PSF_ERR_NULL without dG.
 */
psf_status psf_causal_attn_bwd_learned(const psf_desc *desc, const void *Q, const void *K, const void *V,
                                       const void *G, const void *dO, void *dQ, void *dK, void *dV,
                                       float *dG, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Forward + backward without running the forward pass twice (for callers that train).
 * psf_causal_attn_fwd_save computes the O of psf_causal_attn_fwd (the same function; where the
 * plain call forms the products of its prefix states in half precision the two agree within
 * the rounding of the storage type, not bit for bit) and leaves in `save`
 * (caller memory, psf_fwd_save_bytes(desc) bytes, 256-byte aligned) what the backward pass would
 * otherwise recompute: the sketches, the block states and the denominators.
 * psf_causal_attn_bwd_saved takes that buffer untouched since, the same Q, K, V, G and the O the
 * forward call wrote, and returns the same gradients as psf_causal_attn_bwd (bit for bit).
 * workspace: psf_bwd_workspace_bytes(desc) as for psf_causal_attn_bwd.  Available where
 * psf_bwd_kernel_path(desc) == 3; elsewhere psf_fwd_save_bytes is 0 and the calls return
 * PSF_ERR_UNSUPPORTED (use psf_causal_attn_fwd / psf_causal_attn_bwd there).
 * psf_causal_attn_bwd_saved_learned: the same for desc->learned = 1 with the gradient of the
 * networks' parameters as one more output (dG as for psf_causal_attn_bwd_learned, whose result it
 * equals bit for bit); psf_causal_attn_bwd_saved itself treats the parameters as constants.
 */
size_t psf_fwd_save_bytes(const psf_desc *desc);
psf_status psf_causal_attn_fwd_save(const psf_desc *desc, const void *Q, const void *K, const void *V,
                                    const void *G, void *O, void *save, size_t save_bytes,
                                    void *hip_stream);
psf_status psf_causal_attn_bwd_saved(const psf_desc *desc, const void *Q, const void *K, const void *V,
                                     const void *G, const void *O, const void *dO, void *dQ, void *dK,
                                     void *dV, void *save, size_t save_bytes, void *workspace,
                                     size_t workspace_bytes, void *hip_stream);
psf_status psf_causal_attn_bwd_saved_learned(const psf_desc *desc, const void *Q, const void *K, const void *V,
                                             const void *G, const void *O, const void *dO, void *dQ, void *dK,
                                             void *dV, float *dG, void *save, size_t save_bytes, void *workspace,
                                             size_t workspace_bytes, void *hip_stream);

/*
 * Token-by-token evaluation (the recurrent form behind the paper's remark, Section 5, that the
 * state kept for generation does not grow with the context).  psf_decode_step consumes q, k, v
 * of position `pos` ([batch, heads, 1, d | dv], device, desc->dtype) and writes row `pos` of
 * psf_causal_attn_fwd's output for the sequence fed so far ([batch, heads, 1, dv]): the prefix
 * state Z_l of Section 3.1 over the completed blocks plus the weights of Section 3.2 (or 3.1)
 * inside the current block of desc->b tokens, whose keys are folded into the state when the
 * block completes.  desc->n is the longest context (pos < n); positions must be fed in order
 * 0, 1, 2, ... after psf_decode_reset.
 *   state: device memory of psf_decode_state_bytes(desc) bytes, 256-byte aligned, owned by the
 *   caller: per unit the fp32 state -- r (r + 1) / 2 rows of dv + 1 columns: phi'(x) = m (x) m is
 *   symmetric in its two indices, so only the pairs a <= b' of Z are kept, the off-diagonal ones
 *   doubled; for PSF_BF16 also a bf16 copy of its value columns, rounded from the fp32 state each
 *   time a block is folded in, which is what the steps read -- and the current block's keys,
 *   values and sketches; its size does not depend on n.
 * PSF_FEAT_SKETCH only (PSF_FEAT_EXACT returns PSF_ERR_UNSUPPORTED).  Nothing is allocated and
 * nothing synchronises; everything is enqueued on hip_stream.
 */
size_t psf_decode_state_bytes(const psf_desc *desc);
psf_status psf_decode_reset(const psf_desc *desc, void *state, size_t state_bytes, void *hip_stream);
psf_status psf_decode_step(const psf_desc *desc, const void *q, const void *k, const void *v,
                           const void *G, int32_t pos, void *state, size_t state_bytes, void *o,
                           void *hip_stream);

/*
 * Hand-over from a prompt to token-by-token evaluation.  psf_decode_prefill leaves `state` as
 * if the first n_prompt positions had gone through psf_decode_step one by one (the state is
 * reset first; the next call is psf_decode_step with pos = n_prompt): the keys of the completed
 * blocks folded into the prefix state of Section 3.1, the rest of the prompt in the block
 * cache.  It produces no output rows: those of the prompt are what psf_causal_attn_fwd
 * returns for it.
 *   K [batch, heads, n_prompt, d], V [batch, heads, n_prompt, dv]: device, desc->dtype;
 *   0 <= n_prompt <= desc->n (else PSF_ERR_SHAPE); G as for psf_decode_step.
 *   workspace: psf_decode_prefill_workspace_bytes(desc, n_prompt) bytes of device memory,
 *   256-byte aligned (null allowed when that is zero).  For bf16 storage with d = dv in
 *   {64, 128}, r in {32, 64}, p in {4, 8} (learned sketches: p = 4 and d = 64) and at least one
 *   complete block whose tokens are a multiple of 256 -- whatever b % 256 and the in-block rule
 *   are -- the complete blocks of the prompt go through the forward path's sketch and state
 *   kernels (their buffers are the workspace; K, V and G must then be 16-byte aligned, else
 *   PSF_ERR_ALIGNMENT) and the state starts from their bf16 result, as the forward pass's own
 *   prefix states do; learned sketches need the fp32 sketches of all prompt keys; otherwise
 *   the workspace is empty and the prompt is folded block by block.
 * Nothing is allocated and nothing synchronises; everything is enqueued on hip_stream.
 */
size_t psf_decode_prefill_workspace_bytes(const psf_desc *desc, int32_t n_prompt);
psf_status psf_decode_prefill(const psf_desc *desc, const void *K, const void *V, const void *G,
                              int32_t n_prompt, void *state, size_t state_bytes, void *workspace,
                              size_t workspace_bytes, void *hip_stream);

/*
 * Measurement aid (not part of the attention path): launches `workgroups` workgroups of four
 * wavefronts, each wavefront issuing iters x 8 independent v_mfma_f32_32x32x16_bf16 on non-zero
 * operands, i.e. workgroups x 4 x iters x 8 x 32768 flops in all.  A benchmark times it with
 * events on `hip_stream` to print the rate the matrix cores of this GPU sustain under load
 * beside the published peak.  sink: device memory of at least workgroups x 256 floats (written).
 * Nothing is allocated and nothing synchronises.
 */
psf_status psf_probe_mfma_loop(int32_t workgroups, int32_t iters, void *sink, void *hip_stream);

const char *psf_status_string(psf_status status);

#ifdef __cplusplus
}
#endif
#endif /* PSF_H */
