/*
 * oases.h -- C ABI of the MI355X (gfx950) hot path of Oases: one tensor-model-parallel (TMP)
 * rank's share of a pre-LN GPT transformer layer, forward and backward, run under the
 * sub-batch schedule of the paper's Algorithm 1.
 *
 * Conventions (all entry points)
 *   - Every data pointer is a DEVICE pointer owned by the caller; the library never
 *     allocates, frees or keeps device memory.  `oases_layer_cfg`, `oases_weights`,
 *     `oases_grads`, `oases_peer_sums` and out-parameters are HOST memory.
 *   - Streams are `hipStream_t` passed as `void*` (NULL = the default stream).  Calls only
 *     enqueue work; they never synchronise the host with the device.
 *   - Return value: 0 on success, a negative `OASES_E*` code otherwise; the text of the last
 *     failure of the calling thread is returned by `oases_last_error()`.  Nothing throws or
 *     aborts across this boundary.  Calls on one handle are not thread-safe.
 *   - Notation (paper Sec. II / V; sizes are UNSHARDED unless marked "local"):
 *       b batch, s sequence, h hidden, nh heads, d = h/nh, t TMP degree, r rank in [0,t),
 *       hp = h/t (local attention width = nh/t heads), fp = 4h/t (local FFN columns),
 *       M = b*s tokens, n = number of sub-batches, Ms = M/n rows per sub-batch.
 *     Token rows are batch-major: row = batch_index*s + position.  Sub-batch j owns rows
 *     [j*Ms, (j+1)*Ms).  If n > b a sub-batch is a chunk of one sequence (causal only).
 *   - Tensor layouts, all row-major and 16-byte aligned:
 *       x, y, dy, dx           [M, h]   fp32   residual stream
 *       wqkv                   [h, 3hp] bf16   columns = [Q heads | K heads | V heads] of rank r
 *       bqkv                   [3hp]    fp32
 *       wo                     [hp, h]  bf16   rows of the unsharded projection owned by rank r
 *       w1 / b1                [h, fp] bf16 / [fp] fp32   columns owned by rank r
 *       w2                     [fp, h]  bf16   rows owned by rank r
 *       bo, b2, ln*_g, ln*_b   [h]      fp32   replicated on every rank
 *       gradients              fp32, same shapes as the parameter, ACCUMULATED INTO (+=)
 *       peer sums              [M, h]   fp32   sum over the OTHER t-1 ranks of their partial result
 *                                              at one reduction point
 */
#ifndef OASES_H
#define OASES_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  OASES_OK = 0,
  OASES_EINVAL = -1,     /* bad configuration or argument value */
  OASES_ENULL = -2,      /* required pointer is NULL */
  OASES_EALIGN = -3,     /* device pointer not 16-byte aligned */
  OASES_EWORKSPACE = -4, /* the problem needs more scratch memory than the call has */
  OASES_EHIP = -5,       /* a HIP runtime call failed; text in oases_last_error() */
  OASES_EINFEASIBLE = -6 /* planner: no strategy satisfies the constraints */
};

/* Layer and schedule configuration.  The layer is a pre-LN GPT block: attention block then FFN
 * (paper Sec. II "Large-scale model architecture", Fig. 1), partitioned Megatron-style (Sec. II
 * "Tensor model parallelism": QKV and FC1 by column, projection and FC2 by row). */
typedef struct oases_layer_cfg {
  int32_t hidden, n_heads, seq, batch; /* h, nh, s, b (unsharded) */
  int32_t tp_degree, tp_rank;          /* t, r */
  int32_t n_sub;                       /* sub-batches of the schedule (Alg. 1 uses 2), >= 1 */
  int32_t n_layers;                    /* stacked layers, >= 1 */
  int32_t causal;                      /* 1: key j visible to query i iff j <= i */
  float dropout_p;                     /* hidden-dropout probability, [0,1) */
  uint64_t seed;                       /* Philox key of the dropout masks */
  float ln_eps;                        /* LayerNorm epsilon; 0 selects 1e-5 */
  int32_t flags;                       /* OASES_FLAG_* */
  int32_t arch;                        /* OASES_ARCH_GPT (0), OASES_ARCH_LLAMA or OASES_ARCH_BERT */
  int32_t ffn_hidden;                  /* unsharded inner width F of the FFN; 0 selects 4h (OASES_ARCH_GPT requires 0 or 4h) */
  float rope_theta;                    /* base of the rotary embedding (OASES_ARCH_LLAMA); 0 selects 10000 */
  float attn_dropout_p;                /* dropout on the attention probabilities, [0,1), quantised to round(256 p)/256; any arch */
} oases_layer_cfg;

/* Layer families (the model rows of the paper's Table III).
 * OASES_ARCH_GPT: pre-LayerNorm block, GeLU FFN of width 4h, biases on the four linear maps.
 * OASES_ARCH_LLAMA: pre-RMSNorm block (ln1_g / ln2_g are the RMSNorm weights), rotary embedding on Q and K
 *   ("rotate-half" pairing: element i of a head with element i + d/2, angle pos * theta^(-2i/d), pos = index of the
 *   token in its sequence), SwiGLU FFN f = silu(v2 Wg) * (v2 Wu) of inner width F, no biases.  With fp = F/t
 *   (fp % 32 == 0) the members of oases_weights / oases_grads mean: w1 [h, 2fp] bf16 = this rank's gate and up
 *   columns interleaved in blocks of 32 (columns [64k, 64k+32) = gate columns [32k, 32k+32), the next 32 = the same up
 *   columns), w2 [fp, h]; ln1_b, bqkv, bo, ln2_b, b1, b2 are unused and may be NULL.  The same Megatron partition,
 *   the same four reduction points, schedule, flags and peer sums as OASES_ARCH_GPT.
 * OASES_ARCH_BERT: post-LayerNorm block (the original Transformer / BERT arrangement; set causal = 0 for BERT):
 *   s1 = x + dropout(attention(x) Wo + bo), x1 = LN(s1; ln1_g, ln1_b); s2 = x1 + dropout(gelu(x1 W1 + b1) W2 + b2),
 *   y = LN(s2; ln2_g, ln2_b).  Parameters, shapes, partition and reduction points as OASES_ARCH_GPT. */
enum { OASES_ARCH_GPT = 0, OASES_ARCH_LLAMA = 1, OASES_ARCH_BERT = 2 };

enum {
  OASES_FLAG_SERIALISE = 1, /* enqueue everything on stream_compute only (same results) */
  OASES_FLAG_PROFILE = 2,   /* bracket every operator with timing events, see oases_profile_read */
  OASES_FLAG_RECOMPUTE = 4, /* fine-grained recomputation (paper Sec. IV-B): keep only the input of each computation
                               sequence (x, x1) per layer, rebuild u, qkv, attention output, LSE, v2, pre, f inside
                               oases_backward with the forward kernels -- never a reduction point -- interleaved with
                               the backward operators of the same sub-batch (Alg. 1 "At Backward"); the rebuilt
                               activations share one region of the workspace across layers; same results, bit for bit */
  OASES_FLAG_PIN_GEMM = 8   /* choose the kernel of every forward / input-gradient GEMM as for a launch over all M token rows
                               instead of the sub-batch's Ms rows: the order in which the fp32 terms of an element are added
                               (k slices, k split between waves) then does not depend on n_sub, and y, dx and the weight
                               gradients are the same bit for bit for every sub-batch count (the invariant of Sec. IV-A:
                               splitting the batch leaves the results unchanged); bias and LayerNorm-parameter gradients,
                               which are summed over row groups of a sub-batch, still differ in the last bits.  Default
                               (flag clear): each launch takes the kernel that is fastest for its own shape, and results
                               for different n_sub agree to fp32 summation order only */
};

typedef struct oases_handle oases_handle; /* opaque; holds host metadata and HIP events only */

typedef struct oases_weights { /* one per layer */
  const void *ln1_g, *ln1_b, *wqkv, *bqkv, *wo, *bo, *ln2_g, *ln2_b, *w1, *b1, *w2, *b2;
} oases_weights;

typedef struct oases_grads { /* one per layer; fp32; accumulated into */
  void *ln1_g, *ln1_b, *wqkv, *bqkv, *wo, *bo, *ln2_g, *ln2_b, *w1, *b1, *w2, *b2;
} oases_grads;

/* What the TMP AllReduce would add to this rank's partial at each of the four reduction points of
 * a layer (Sec. IV-B: y = sum_i x_i).  A NULL member means "no peers at this point". */
typedef struct oases_peer_sums { /* one per layer */
  const void *fwd_attn; /* added to A*Wo_r        -> Z1  */
  const void *fwd_ffn;  /* added to f*W2_r        -> Z2  */
  const void *bwd_ffn;  /* added to dG*W1_r^T     -> dV2 */
  const void *bwd_attn; /* added to dQKV*Wqkv_r^T -> dU  */
} oases_peer_sums;

/* Validate the configuration and plan workspace and schedule.  Pure host code: works without a
 * GPU.  EINVAL if h % nh, nh % t, 4h % t, M % n, d not in {64,128}, r >= t, p outside [0,1),
 * a sub-batch that is neither whole sequences nor an equal chunk of one sequence, or sequence
 * chunks with causal = 0. */
int oases_create(const oases_layer_cfg *cfg, oases_handle **out);
void oases_destroy(oases_handle *h);

/* Bytes of caller-allocated device workspace (activation stash of all layers + backward scratch).
 * The same workspace must be passed to oases_forward and to the oases_backward that follows it; every call that takes
 * a workspace also takes its size in bytes and returns OASES_EWORKSPACE, before any launch, if that is less than this. */
size_t oases_workspace_bytes(const oases_handle *h);

/* Forward of all layers under Alg. 1 "At Forward": for each computation sequence, sub-batch after
 * sub-batch; after each row-parallel GEMM the reduction point of that sub-batch is started on
 * stream_comm (adds the peer sum, then the fused bias+dropout+residual(+LayerNorm) that consumes it)
 * while stream_compute goes on with the next sub-batch.  w: [n_layers]; peers: [n_layers] or NULL.
 * x [M,h] fp32 in, y [M,h] fp32 out (y may not alias x). */
int oases_forward(oases_handle *h, const oases_weights *w, const void *x, void *y,
                  const oases_peer_sums *peers, void *workspace, size_t workspace_bytes,
                  void *stream_compute, void *stream_comm);

/* Backward of all layers under Alg. 1 "At Backward" with stored activations: sub-batches in
 * reverse order; each column-parallel input-gradient partial starts its reduction point on
 * stream_comm, under which the next sub-batch's GEMMs run; the weight-gradient GEMMs of a block, on which no
 * reduction depends, run once over the rows of all sub-batches behind the last reduction start.
 * x: the input given to oases_forward (read again by the first LayerNorm's backward);
 * dy [M,h] fp32 in, dx [M,h] fp32 out; g: [n_layers], accumulated into. */
int oases_backward(oases_handle *h, const oases_weights *w, const void *x, const void *dy,
                   void *dx, const oases_grads *g, const oases_peer_sums *peers, void *workspace,
                   size_t workspace_bytes, void *stream_compute, void *stream_comm);

/* Segment-level calls: lock-step emulation of the t ranks of a partition on one GPU.  What rank r feeds into its FFN block
 * depends on the other ranks' attention partials, so t ranks can only be run side by side one computation sequence at a
 * time: each rank (its own handle, weights and workspace) runs a segment up to its reduction point, the caller forms
 * y = sum_i x_i over the ranks' partials (the AllReduce of Sec. IV-B, whose input gradient is its output gradient, Eq. (1))
 * and hands the sum to every rank's next segment.  A segment runs the operators of ONE layer for ALL sub-batches, in the
 * order of oases_schedule_dump, on one stream.
 *   forward  segment 0: [LN1 (first layer), QKV, attention, projection]              ends in   Z1_r  (fwd_attn point)
 *            segment 1: [bias+dropout+residual+LN2 on Z1, FC1+GeLU, FC2]             Z1 in,    ends in Z2_r (fwd_ffn point)
 *            segment 2: [bias+dropout+residual on Z2 (+ LN1 of the next layer)]      Z2 in,    writes the layer output
 *   backward segment 2: [dropout backward of dy]  (top layer only; below it this work belongs to segment 3 of the layer above)
 *            segment 1: [FC2 and FC1 input gradients, their weight gradients]        ends in   dV2_r (bwd_ffn point)
 *            segment 0: [LN2 backward + residual + dropout backward on dV2, projection / attention / QKV gradients]
 *                                                                                     dV2 in,   ends in dU_r (bwd_attn point)
 *            segment 3: [LN1 backward + residual on dU]                               dU in,    writes dx (or the layer below's dy)
 * Forward: layers bottom-up, segments 0, 1, 2; backward: layers top-down, segments 2 (top layer), 1, 0, 3.
 * partial_out: device [M,h] fp32 that receives the partial the segment ends in, or NULL (it then stays in the workspace
 *   tensor "z1" / "z2" / "dv2" / "du", see oases_workspace_tensor); EINVAL if given for a segment that ends in none.
 * reduced_in: device [M,h] fp32, the REDUCED tensor (sum over all ranks, this rank's partial included) the segment starts
 *   from, or NULL to read this rank's own partial from the workspace (t = 1); EINVAL if given for a segment that starts
 *   from none.  x, y, dy, dx, w, g, workspace as in oases_forward / oases_backward (the same workspace through all
 *   segments of a step); peer sums do not exist at this level.  Run back to back with NULL partial_out / reduced_in the
 *   segments give what oases_forward / oases_backward give without peer sums: y, dx and the weight-matrix gradients bit for
 *   bit; the bias and LayerNorm-parameter gradients (column sums, which a segment finishes at once and the whole pass
 *   finishes in one launch at its end) up to the order of the fp32 additions. */
int oases_forward_segment(oases_handle *h, int layer, int segment, const oases_weights *w, const void *x, void *y,
                          void *workspace, size_t workspace_bytes, void *partial_out, const void *reduced_in,
                          void *stream);
int oases_backward_segment(oases_handle *h, int layer, int segment, const oases_weights *w, const void *x,
                           const void *dy, void *dx, const oases_grads *g, void *workspace, size_t workspace_bytes,
                           void *partial_out, const void *reduced_in, void *stream);

/* The operator order of the schedule as text, one operator per line
 * ("<stream> <op> L<layer> sb<sub-batch>", "sb*" = all sub-batches at once), NUL-terminated into buf (at most n bytes).
 * Returns the number of bytes the full text needs (like snprintf).  Host only. */
int oases_schedule_dump(const oases_handle *h, int backward, char *buf, size_t n);

/* Byte offset and size inside the workspace of a named stashed tensor of one layer, for tests and
 * debugging.  Names: "u","qkv","attn","lse","z1","x1","v2","pre","f","z2","mu1","rstd1","mu2",
 * "rstd2","dz2","dg","dv2","dx1","dz1","da","dqkv","du".  EINVAL for an unknown name. */
int oases_workspace_tensor(const oases_handle *h, const char *name, int layer, size_t *offset,
                           size_t *bytes);

/* Per-operator timers (the paper's offline profiling records each operation's time with dedicated
 * timers, Sec. V "Implementation"): with OASES_FLAG_PROFILE set at creation, every operator of the last
 * oases_forward (backward = 0) or oases_backward (backward = 1) call is bracketed by HIP events on its
 * stream.  This call waits for those events and writes the elapsed milliseconds of the first n operators,
 * in the order of oases_schedule_dump, to HOST array ms.  Returns the number of operators of the pass,
 * or a negative error (EINVAL if the flag was not set or the pass has not run). */
int oases_profile_read(oases_handle *h, int backward, float *ms, int n);

const char *oases_last_error(void); /* thread-local, never NULL */

/* ---------------------------------------------------------------------------------------------
 * Single-operator entry points: the kernels of the path, one at a time (used by the per-operator
 * parity tests and the per-kernel roofline measurements).  Same conventions as above.
 * ------------------------------------------------------------------------------------------- */

/* Keep mask of hidden dropout as bytes (1 keep, 0 drop) for global rows row0..row0+rows-1 of the
 * unsharded [M,h] activation: element e = row*h+col takes word (e mod 4) of Philox4x32-10 with key
 * (seed lo, seed hi) and counter (e/4 lo, e/4 hi, site, layer); keep iff (word >> 8) >= round(p*2^24). */
int oases_op_dropout_mask(uint8_t *mask, uint64_t seed, int layer, int site, int64_t row0,
                          int rows, int h, float p, void *stream);

/* LayerNorm forward over rows of x [rows,h] fp32: out bf16 [rows,h], mu/rstd fp32 [rows]. */
int oases_op_layernorm_fwd(const void *x, const void *gamma, const void *beta, void *out, void *mu,
                           void *rstd, int rows, int h, float eps, void *stream);

/* Reduction point + bias + dropout + residual (+ LayerNorm):
 *   xo = xin + keep * (part + peer + bias) / (1-p);  if ln_out: ln_out = LN(xo) (bf16), mu, rstd.
 * part, xin, xo fp32 [rows,h]; peer may be NULL; ln_out/gamma/beta/mu/rstd may all be NULL. */
int oases_op_bias_dropout_residual_ln(const void *part, const void *peer, const void *bias,
                                      const void *xin, void *xo, const void *gamma,
                                      const void *beta, void *ln_out, void *mu, void *rstd,
                                      int rows, int h, float eps, uint64_t seed, int layer,
                                      int site, int64_t row0, float p, void *stream);

/* Backward of dropout+bias at a forward reduction point:
 *   dz = keep * dyin / (1-p) -> bf16 [rows,h];  dbias[h] += column sums of dz (fp32 values). */
int oases_op_dropout_bwd(const void *dyin, void *dz, void *dbias, int rows, int h, uint64_t seed,
                         int layer, int site, int64_t row0, float p, void *scratch,
                         void *stream);

/* LayerNorm backward + residual (+ reduction point, + dropout backward of the layer input side):
 *   g = part + peer;  dxo = dres + LN'(g; x, mu, rstd, gamma);  dgamma += , dbeta += ;
 *   if dz: dz = keep * dxo / (1-p) (bf16), dbias += column sums of dz.
 * part/peer/dres/x/dxo fp32 [rows,h]; peer, dz, dbias may be NULL.  scratch: fp32 [3*1024*h]. */
int oases_op_layernorm_bwd(const void *part, const void *peer, const void *dres, const void *x,
                           const void *mu, const void *rstd, const void *gamma, void *dxo,
                           void *dgamma, void *dbeta, void *dz, void *dbias, int rows, int h,
                           uint64_t seed, int layer, int site, int64_t row0, float p,
                           void *scratch, void *stream);

/* RMSNorm counterparts (the LLaMA layers of the paper's Table III): y = gamma * x * rstd, rstd = 1/sqrt(mean(x^2)+eps);
 * no mean, no beta, no bias at the reduction point.  Shapes and optional arguments as for the LayerNorm entry
 * points above; scratch of the backward: fp32 [3*1024*h]. */
int oases_op_rmsnorm_fwd(const void *x, const void *gamma, void *out, void *rstd, int rows, int h,
                         float eps, void *stream);
/*   xo = xin + keep * (part + peer) / (1-p);  if ln_out: ln_out = RMSNorm(xo) (bf16), rstd. */
int oases_op_dropout_residual_rmsnorm(const void *part, const void *peer, const void *xin, void *xo,
                                      const void *gamma, void *ln_out, void *rstd, int rows, int h,
                                      float eps, uint64_t seed, int layer, int site, int64_t row0,
                                      float p, void *stream);
/*   g = part + peer;  dxo = dres + RMSNorm'(g; x, rstd, gamma);  dgamma += ;  if dz: dz = keep * dxo / (1-p) (bf16). */
int oases_op_rmsnorm_bwd(const void *part, const void *peer, const void *dres, const void *x,
                         const void *rstd, const void *gamma, void *dxo, void *dgamma, void *dz,
                         int rows, int h, uint64_t seed, int layer, int site, int64_t row0, float p,
                         void *scratch, void *stream);

/* Rotary position embedding.  table: fp32 [seq][head_dim/2][2] = (cos, sin) of pos * theta^(-2i/head_dim), written
 * by oases_op_rope_table (angles in fp64).  oases_op_rope rotates, in place, the pair (i, i + head_dim/2) of every
 * head of the Q and K parts of qkv [rows, ld] bf16 = [Q heads | K heads | V heads] by the angle of the token's
 * position (row0 + row) mod seq; inverse != 0 rotates back (what the gradients of Q and K need).  head_dim % 16 == 0. */
int oases_op_rope_table(void *table, int seq, int head_dim, float theta, void *stream);
int oases_op_rope(void *qkv, int ld, int rows, int64_t row0, int seq, int heads, int head_dim,
                  const void *table, int inverse, void *stream);

/* GEMM family on bf16 operands with fp32 accumulation.  `op`:
 *   OASES_GEMM_NN  C[M,N]  = A[M,K] * B[K,N]            (forward of a linear map)
 *   OASES_GEMM_NT  C[M,N]  = A[M,K] * B[N,K]^T          (input gradient)
 *   OASES_GEMM_TN  C[M,N] += A[K,M]^T * B[K,N]          (weight gradient, C fp32)
 * `epi` (NN/NT): OASES_EPI_F32 C fp32; OASES_EPI_BF16 C bf16; OASES_EPI_BIAS_BF16 C = acc+bias (bf16);
 *   OASES_EPI_BIAS_GELU aux = acc+bias (bf16, "pre"), C = GeLU_tanh(acc+bias) (bf16);
 *   OASES_EPI_DGELU C = acc * GeLU_tanh'(aux) (bf16), aux = stored "pre" [M,N] bf16.
 *   OASES_EPI_SWIGLU (NN only, N % 64 == 0): the N columns of B are the gate and up projections of a SwiGLU block
 *     interleaved in blocks of 32: columns [64k, 64k+32) = gate columns [32k, 32k+32), [64k+32, 64k+64) = the same
 *     up columns.  aux [M,N] bf16 = acc (gate and up pre-activations, same interleaving, ldaux >= N);
 *     C [M,N/2] bf16 = silu(gate) * up, ldc >= N/2.  Never runs over k slices.
 *   OASES_EPI_DSWIGLU (NT only, N % 32 == 0): acc = dF [M,N]; aux [M,2N] = the stored pre-activations (layout
 *     above); C [M,2N] bf16 = [dF * up * silu'(gate) | dF * silu(gate)] in the same interleaving, ldc >= 2N.
 * lda/ldb/ldc are row strides in elements.  M,N,K must be multiples of 8; EINVAL otherwise.
 * workspace (optional, fp32 scratch of workspace_bytes): lets tile-starved shapes split K -- slices write fp32
 * partial planes [slices][M][N] that a second kernel adds in slice order before the epilogue (deterministic).
 * NULL: never split. */
enum { OASES_GEMM_NN = 0, OASES_GEMM_NT = 1, OASES_GEMM_TN = 2 };
enum { OASES_EPI_F32 = 0, OASES_EPI_BF16 = 1, OASES_EPI_BIAS_BF16 = 2, OASES_EPI_BIAS_GELU = 3,
       OASES_EPI_DGELU = 4, OASES_EPI_SWIGLU = 6, OASES_EPI_DSWIGLU = 7 };
int oases_op_gemm(int op, int epi, int M, int N, int K, const void *A, int lda, const void *B,
                  int ldb, void *C, int ldc, const void *bias, void *aux, int ldaux,
                  void *workspace, size_t workspace_bytes, void *stream);

/* Which kernel instantiation oases_op_gemm launches for a problem given workspace_bytes of split-K scratch:
 * returns 100000000*W + 1000000*slices + 1000*BM + BN, or EINVAL.  BM x BN: block tile; slices: k slices with fp32
 * partial planes in the workspace; W = 1 if the waves of a workgroup split the k steps of a stage between them
 * (rectangular tiles only), e.g. 101128256 = 128x256 tiles, waves split k, one slice; W = 2 names the kernels that
 * load their operand tiles from global memory straight into LDS: 201256256 (256x256 tiles, four LDS stages of 32 k
 * columns; K % 32 == 0; an operand whose k index is the contiguous one -- A of NN and NT, B of NT -- must fill its tiles:
 * M resp. N % 256 == 0) and 201128256 (128x256 tiles, three LDS stages of 64 k columns, waves split k; K % 64 == 0;
 * any M, N the GEMM accepts; no forward SwiGLU epilogue; also over 2 or 4 k slices of whole stages, 202128256 and
 * 204128256, K % (64 * slices) == 0); the 256x256 kernel takes one slice only.  W = 3 names the eight-wave forms of
 * the same tiles (two waves per SIMD that alternate between loading and multiplying): 301256256, 301128256, 302128256,
 * 304128256, on the shapes of their W = 2 counterparts; 301128256 gives bit for bit what 201128256 gives.  The W = 2 and
 * W = 3 kernels address an operand with 32-bit byte offsets: oases_op_gemm launches them only if rows x leading
 * dimension x 2 bytes of A and of B stay under 2 GiB (the staged kernel of the same tile otherwise), and
 * oases_op_gemm_forced returns EINVAL for them on larger operands.
 * Host only; used to group per-operator timings by kernel. */
int oases_op_gemm_variant(int op, int epi, int M, int N, int K, size_t workspace_bytes);
/* oases_op_gemm on the instantiation `variant` names (encoding above) instead of the one the library would choose:
 * for tests and tuning sweeps.  EINVAL if no such instantiation exists (block tiles 256x256, 128x256, 256x128,
 * 128x128; W = 1 only with the rectangular ones; W = 2, 3 only as x01256256, x01128256, x02128256 or x04128256 on shapes they fit; 1..8 slices), if the slices do not fit K (every slice needs at least
 * one k column) or if the workspace is smaller than slices*M*N*4 bytes.  Results of different variants differ only
 * by the fp32 summation order. */
int oases_op_gemm_forced(int variant, int op, int epi, int M, int N, int K, const void *A, int lda,
                         const void *B, int ldb, void *C, int ldc, const void *bias, void *aux,
                         int ldaux, void *workspace, size_t workspace_bytes, void *stream);
/* Two weight-gradient contractions over the same K token rows in ONE launch of the eight-wave 128x256 direct-to-LDS kernel:
 *   C0 [M0,N0] += A0^T B0   and   C1 [M1,N1] += A1^T B1,   A_i bf16 [K, lda_i >= M_i], B_i bf16 [K, ldb_i >= N_i],
 *   C_i fp32 [M_i, ldc_i >= N_i] (accumulated into, as the TN form of oases_op_gemm does); all device pointers,
 * 16-byte aligned; lda, ldb multiples of 8, ldc of 4.  The tiles of the second problem follow those of the first in the
 * grid, so that two launches that would each leave CUs idle (or need k slices to fill them) share one round of
 * workgroups: the backward pass issues the attention block's two weight gradients (Sec. II: projection and QKV) this way
 * when oases_op_gemm_tn_pair_wins says so.  Needs whole tiles, M_i % 128 == 0, N_i % 256 == 0, and K % 64 == 0: EINVAL
 * otherwise, before any launch.  Each C_i gets exactly what oases_op_gemm_forced(301128256, TN, ...) gives it. */
int oases_op_gemm_tn_pair(int K, int M0, int N0, const void *A0, int lda0, const void *B0, int ldb0, void *C0,
                          int ldc0, int M1, int N1, const void *A1, int lda1, const void *B1, int ldb1, void *C1,
                          int ldc1, void *stream);
/* Host only: 1 if the library issues two such weight gradients as one launch (both fit whole 128x256 tiles, more than 128
 * tiles together, and fewer rounds of 256 workgroups together than apart), else 0. */
int oases_op_gemm_tn_pair_wins(int K, int M0, int N0, int M1, int N1);
/* Bytes of split-K scratch that oases_forward / oases_backward set aside inside the workspace. */
size_t oases_gemm_workspace_bytes(const oases_handle *h);

/* Column sums of a bf16 matrix [rows, cols] (row stride ld) accumulated into fp32 out[cols].
 * scratch: fp32 [1024*cols]. */
int oases_op_colsum_bf16(const void *a, int ld, int rows, int cols, void *out, void *scratch,
                         void *stream);

/* oases_op_colsum_bf16 for callers that cannot allocate device memory or carry a scratch buffer (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the partial-sum rows between the two kernels live in
 * a 16 MiB device array inside the library (one per GPU, held until the process ends) instead of `scratch`; the call
 * allocates nothing.  Same kernels, same result bit for bit.  cols <= 4096, else OASES_EWORKSPACE before any launch.
 * All calls on one GPU share that array: calls that may overlap on one GPU (different streams, different host
 * threads) race; calls on one stream are ordered and safe. */
int oases_op_colsum_bf16_static(const void *a, int ld, int rows, int cols, void *out, void *stream);

/* Flash-style attention over the local heads.  qkv [batch*seq, 3*hp] bf16 with hp = heads*d and
 * columns [Q | K | V]; queries are the rows row0..row0+rows-1 (a whole number of sequences, or a chunk
 * of one sequence when causal).  Keys/values of the same sequence are read from qkv at any row.
 * out [batch*seq, hp] bf16 (only the query rows are written); lse [batch, heads, seq] fp32 holds
 * log-sum-exp of the scaled scores (natural log). */
int oases_op_attention_fwd(const void *qkv, void *out, void *lse, int batch, int seq, int heads,
                           int head_dim, int causal, int row0, int rows, void *stream);

/* Attention backward for the rows row0..row0+rows-1: writes dq, dk, dv (bf16) for those rows into
 * dqkv [batch*seq, 3*hp].  dk/dv of a row sum over every query of its sequence that sees it, so dout
 * (and out, lse) must already hold the rows of all such queries.  delta: fp32 scratch
 * [batch, heads, seq]; this call fills it for the query rows it needs. */
int oases_op_attention_bwd(const void *qkv, const void *out, const void *dout, const void *lse,
                           void *delta, void *dqkv, int batch, int seq, int heads, int head_dim,
                           int causal, int row0, int rows, void *stream);

/* The same two operators with dropout on the attention probabilities (the layer's attn_dropout_p): A = (D o P) V / (1-p'),
 * p' = T/256, T = round(256 p).  The mask D is a function of (sequence b, global head = head0 + local head, query
 * position q, key position k), independent of partition and sub-batch split: the 4 x 4 block (q div 4, k div 4) draws
 * one Philox4x32-10 output with key (seed lo, seed hi) and counter (k div 4, q div 4, b*heads_total + head,
 * layer | 2^31); element (q, k) is kept iff byte (k mod 4), low byte first, of word (q mod 4) is >= T.  The backward
 * regenerates the mask.  T == 0 runs the kernels without dropout.  EINVAL if head0 + heads > heads_total. */
int oases_op_attention_dropout_fwd(const void *qkv, void *out, void *lse, int batch, int seq, int heads,
                                   int head_dim, int causal, int row0, int rows, uint64_t seed, int layer,
                                   float p, int head0, int heads_total, void *stream);
int oases_op_attention_dropout_bwd(const void *qkv, const void *out, const void *dout, const void *lse,
                                   void *delta, void *dqkv, int batch, int seq, int heads, int head_dim,
                                   int causal, int row0, int rows, uint64_t seed, int layer, float p,
                                   int head0, int heads_total, void *stream);

/* Measurement helper for the roofline the GEMMs are priced against (no step of the path): every wave of `workgroups`
 * 256-thread workgroups issues iters x 8 register-resident v_mfma_f32_32x32x16_bf16 (2 * 32*32*16 flop each) on 8
 * independent accumulators, with no memory traffic; random_operands = 0: all-zero operands, 1: pseudo-random, roughly
 * normal bf16 operands (on a power-capped part the sustained clock, and so the rate, depends on the operand values).
 * out: device fp32 [workgroups * 256], written once per thread.  The caller times the launch:
 * flop = workgroups * 4 waves * iters * 8 * 32768. */
int oases_probe_mfma_rate(int random_operands, int iters, int workgroups, void *out, void *stream);
/* Measurement helper (no step of the path): the rate at which a workgroup of `waves` (4 or 8) waves pulls data that is
 * resident in its XCD's L2 straight into LDS with 16-byte-per-lane direct-to-LDS loads -- the ceiling over the operand
 * streams of the GEMM kernels.  Workgroup b sweeps bytes [65536 b, 65536 (b+1)) of src (device, 16-byte aligned,
 * src_bytes >= 65536 * workgroups) iters times, each wave 8 KiB per iteration; nothing is read back.  out: device fp32
 * [>= 512], not written in practice.  The caller times the launch: bytes = workgroups * waves * iters * 8192. */
int oases_probe_lds_load_rate(int waves, int iters, int workgroups, const void *src, size_t src_bytes, void *out,
                              void *stream);

#ifdef __cplusplus
}
#endif
#endif /* OASES_H */
