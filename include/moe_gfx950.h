/*
 * moe_gfx950 -- forward pass of the position-wise top-2 Mixture-of-Experts layer
 * of GShard (arXiv 2006.16668) on one AMD MI355X (gfx950), one device's share of
 * tokens.  C ABI; every step runs in hand-written HIP kernels.
 *
 * Notation (paper, Section 2.2 and 3.1):
 *   G groups, S tokens per group, M model dimension, H expert hidden dimension,
 *   E experts, C capacity of one expert inside one group.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller, row-major,
 *     contiguous, 16-byte aligned.  The config struct is a HOST pointer.
 *   - The library allocates nothing, frees nothing and never synchronises the
 *     device.  Scratch memory comes from the caller's workspace (size:
 *     moe_workspace_bytes / moe_gate_workspace_bytes); nothing a call computes
 *     survives it outside the caller's buffers.  The only state the library
 *     keeps is per-device set-up that does not depend on any argument: kernels
 *     that use more than 64 KB of LDS have that limit raised by a host-side
 *     attribute call before their first launch on a device, the number of compute
 *     units is read once, and moe_gate_noalloc looks up the address of its array.
 *     moe_prepare() does all of it for the current device; otherwise the first
 *     call that launches such a kernel does it (thread-safe, idempotent).  A
 *     caller that records a HIP graph calls moe_prepare() (or the entry point
 *     itself once) before starting the capture.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream) and the call returns immediately.
 *   - Return value: MOE_OK or a negative moe_status.  Nothing is enqueued when
 *     an argument check fails.  No exception or abort crosses the boundary.
 *     MOE_EHIP reports what hipPeekAtLastError() says after a launch, so an error
 *     that earlier work of the caller left pending on the host thread is
 *     reported by the next launch here as well; the error itself stays in place
 *     for the caller's own hipGetLastError().
 *   - Activations / expert weights / buffers have the element type
 *     cfg->act_dtype (fp32 or bf16).  The gate path (wg, u, gates, weights,
 *     auxiliary loss) is always fp32.  bf16 expert GEMMs accumulate in fp32; the
 *     hidden activation h is rounded to bf16 once.
 *
 * Slot codes in `slot[G,S,2]`:  >= 0  position c in the expert's buffer;
 *   MOE_SLOT_OVERFLOW (-1) expert already full (Section 2.2, "Expert capacity");
 *   MOE_SLOT_NOT_SAMPLED (-2) second expert skipped by random routing
 *   (Section 2.2, "Random routing"); it takes precedence over -1.
 */
#ifndef MOE_GFX950_H
#define MOE_GFX950_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype;

typedef enum {
  MOE_OK = 0,
  MOE_EINVAL = -1,       /* null / misaligned pointer, non-positive dimension, E < 2, C < 1 */
  MOE_EUNSUPPORTED = -2, /* a shape the kernels do not take: M or H not a multiple of 16 bytes
                            (8 bf16 / 4 fp32 elements), more than 2^30 tokens or 2^31 slots */
  MOE_EWORKSPACE = -3,   /* workspace too small */
  MOE_EHIP = -4          /* a kernel launch failed; hipGetLastError() is left for the caller */
} moe_status;

#define MOE_SLOT_OVERFLOW (-1)
#define MOE_SLOT_NOT_SAMPLED (-2)

typedef struct {
  int32_t G, S, M, H, E, C;
  int32_t act_dtype; /* moe_dtype */
} moe_config;

/* Human-readable name of a status code (static string, never NULL). */
const char* moe_status_string(int status);

/* One-time set-up of the current device (see the conventions above): LDS limits of the
 * kernels, compute-unit count, address of moe_gate_noalloc's array.  Host-side queries and
 * attribute calls only: no allocation, no launch, no synchronisation.  Optional. */
int moe_prepare(void);

/* Bytes of workspace moe_gate needs for this config.  Pure host function. */
int moe_gate_workspace_bytes(const moe_config* cfg, size_t* bytes);

/* Bytes of workspace moe_forward needs (routing tensors, expert buffers and the
 * gate scratch).  Pure host function. */
int moe_workspace_bytes(const moe_config* cfg, size_t* bytes);

/* Bytes of workspace moe_forward_train needs: moe_workspace_bytes plus what only the backward
 * pass reads (the softmax gates [G,S,E] fp32 and one bit per element of h).  Pure host function. */
int moe_train_workspace_bytes(const moe_config* cfg, size_t* bytes);

/*
 * Top2Gating: Algorithm 1 of the paper for G independent groups (Section 2.2,
 * "Local group dispatching") and line 1 of Algorithm 2 (gate softmax).
 *
 *   g[g,s,:]   = softmax_e( sum_m x[g,s,m] wg[m,e] )
 *   (e1,e2)    = indices of the largest and second largest gate (ties: lowest index)
 *   pass 1     : token s takes position #{s'<s : e1[s']=e1[s]} of expert e1,
 *                kept when the position is < C; weight g1/(g1+g2)
 *   l_aux[g]   = (1/E) sum_e (c1[g,e]/S) mean_gate[g,e],  c1 = first-choice counts
 *                (all tokens, also overflowing ones), mean_gate = mean over s of g
 *   pass 2     : second choice sampled iff 2*g2/(g1+g2) > u[g,s]; a sampled token
 *                takes position c1[g,e2] + #{s'<s sampled : e2[s']=e2[s]}, kept when
 *                < C; weight g2/(g1+g2).  A non-sampled second choice consumes no
 *                capacity.
 *
 * in : x [G,S,M] act_dtype;  wg [M,E] fp32;  u [G,S] fp32 uniforms in [0,1)
 * out: expert_idx [G,S,2] i32;  slot [G,S,2] i32 (codes above);
 *      weight [G,S,2] fp32 combine weight, 0 when the choice is not kept;
 *      fill [G,E] i32 occupied slots;  src_token [E,G,C] i32 inverse map
 *      slot -> s (the gather indices of Section 3.2's gather-based dispatch), -1 empty;
 *      c1 [G,E] i32;  mean_gate [G,E] fp32;  aux [G] fp32;
 *      gates_opt [G,S,E] fp32 or NULL (full softmax output, for inspection)
 * ws : at least moe_gate_workspace_bytes(cfg)
 */
int moe_gate(const moe_config* cfg, const void* x, const float* wg, const float* u,
             int32_t* expert_idx, int32_t* slot, float* weight, int32_t* fill,
             int32_t* src_token, int32_t* c1, float* mean_gate, float* aux,
             float* gates_opt, void* ws, size_t ws_bytes, void* stream);

/*
 * The gate weights in the form the logit kernels multiply (Algorithm 2, line 1: the GSM,ME->GSE
 * projection).  bf16 layers compute the logits on the matrix cores with wg split into three bf16
 * terms (hi + mid + lo = all 24 mantissa bits, so every product with a bf16 activation is exact)
 * laid out in the order of the MFMA operand; moe_gate and moe_forward build that form from wg
 * on every call.  wg is a parameter, so a caller can build it once per weight update instead:
 *   moe_gate_pack_bytes   size of the packed form for this config (0: this gate reads wg as it
 *                         is and the calls below take wg_packed == NULL).  Pure host function.
 *   moe_gate_pack         wg [M,E] fp32 -> wg_packed (caller-owned, 256-byte aligned)
 *   moe_gate_prepacked    moe_gate        that reads wg_packed instead of packing wg
 *   moe_forward_prepacked moe_forward_events (events may be NULL) likewise
 * Results are bit-identical to moe_gate / moe_forward with the same wg.  The library keeps no
 * record of the buffer: passing a wg_packed that was built from other weights, or for another
 * config, gives the logits of those weights.
 */
int moe_gate_pack_bytes(const moe_config* cfg, size_t* bytes);
int moe_gate_pack(const moe_config* cfg, const float* wg, void* wg_packed, void* stream);
int moe_gate_prepacked(const moe_config* cfg, const void* x, const float* wg, const void* wg_packed,
                       const float* u, int32_t* expert_idx, int32_t* slot, float* weight,
                       int32_t* fill, int32_t* src_token, int32_t* c1, float* mean_gate,
                       float* aux, float* gates_opt, void* ws, size_t ws_bytes, void* stream);

/*
 * moe_gate for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments (minus ws / ws_bytes), same kernels and bit-identical results; the scratch memory
 * is an array of moe_gate_noalloc_max_bytes() = 16 MiB inside the library's own device image,
 * one copy per GPU, held until the process ends.  The call allocates and frees nothing.
 * Returns MOE_EWORKSPACE (nothing enqueued) when moe_gate_workspace_bytes(cfg) exceeds that
 * size.  All calls on one GPU share that GPU's array: calls that may overlap on one GPU (two
 * streams, two host threads) race; calls on one stream are ordered and safe.  The first call
 * on a device looks the array's address up (a host-side query, no allocation).
 */
int moe_gate_noalloc_max_bytes(size_t* bytes);
int moe_gate_noalloc(const moe_config* cfg, const void* x, const float* wg, const float* u,
                     int32_t* expert_idx, int32_t* slot, float* weight, int32_t* fill,
                     int32_t* src_token, int32_t* c1, float* mean_gate, float* aux,
                     float* gates_opt, void* stream);

/*
 * Dispatch (Algorithm 2, the GSEC,GSM->EGCM einsum, computed as the gather of
 * Section 3.2):  buf[e,g,c,:] = x[g, src_token[e,g,c], :], zeros where
 * src_token is -1.
 * in : x [G,S,M];  src_token [E,G,C]        out: buf [E,G,C,M] act_dtype
 */
int moe_dispatch(const moe_config* cfg, const void* x, const int32_t* src_token,
                 void* buf, void* stream);

/*
 * Expert networks (Eq. 2; Algorithm 2, EGCM,EMH->EGCH, relu, EGCH,EHM->EGCM):
 *   h[e]   = relu( buf[e] . wi[e] )        [G*C, M] x [M, H]
 *   out[e] = h[e] . wo[e]                  [G*C, H] x [H, M]
 * The output keeps the EGCM order on one device (the paper prints GECM, its layout after the
 * reverse exchange between devices).
 * in : buf [E,G,C,M];  wi [E,M,H];  wo [E,H,M]   (act_dtype)
 *      fill [G,E] i32 or NULL: occupied slots per (group, expert) as moe_gate returns them; the
 *      occupied slots of a segment buf[e,g,:,:] are its first fill[g,e] ones
 * tmp: h_ws [E,G,C,H] act_dtype (caller-provided scratch, contents private to the call)
 *      ws  NULL, or moe_expert_ffn_workspace_bytes(cfg) bytes, 256-byte aligned
 * out: out [E,G,C,M] act_dtype
 * Without fill (or without ws) every row of buf is multiplied, occupied or not: an empty row is
 * zero and FFN_e(0) = 0 since the experts have no bias (Section 2.2, "Expert capacity": a
 * buffer position holds a token or nothing).  With fill and ws, and when
 * moe_forward_packs_rows(cfg) says the kernels take the shape, only the occupied slots are
 * multiplied: the kernels pack each expert's occupied rows to the front of its block (row maps
 * in ws), multiply whole 256-row tiles of them and store each result row at its slot of out;
 * the slots c >= fill[g,e] of out are then NOT written (combine never reads them).  Occupied
 * rows get bit-identical results either way.
 */
int moe_expert_ffn_workspace_bytes(const moe_config* cfg, size_t* bytes);
int moe_expert_ffn(const moe_config* cfg, const void* buf, const int32_t* fill, const void* wi,
                   const void* wo, void* h_ws, void* out, void* ws, size_t ws_bytes, void* stream);

/*
 * Combine (Eq. 3; Algorithm 2, the GSEC,EGCM->GSM einsum, computed as a gather):
 *   y[g,s,:] = sum_{k: slot[g,s,k] >= 0} weight[g,s,k] * out[expert_idx[g,s,k], g, slot[g,s,k], :]
 * A token with no kept choice gets a zero row (Section 2.2: overflowed tokens).
 * Accumulation in fp32, one rounding to act_dtype.
 */
int moe_combine(const moe_config* cfg, const void* out, const int32_t* expert_idx,
                const int32_t* slot, const float* weight, void* y, void* stream);

/*
 * The whole layer forward (Algorithm 2): gate -> dispatch -> experts -> combine.
 * in : x [G,S,M], wg [M,E], u [G,S], wi [E,M,H], wo [E,H,M]
 * out: y [G,S,M] act_dtype;  aux [G] fp32 (per-group auxiliary loss)
 * ws : at least moe_workspace_bytes(cfg); all routing tensors and expert buffers
 *      live there and are overwritten by every call.
 */
int moe_forward(const moe_config* cfg, const void* x, const float* wg, const float* u,
                const void* wi, const void* wo, void* y, float* aux,
                void* ws, size_t ws_bytes, void* stream);

/*
 * Whether moe_forward folds the dispatch into the first expert GEMM for this config
 * (Section 3.2's gather form: the GEMM's operand copies pick the rows of x through
 * src_token, and the [E,G,C,M] buffer is never written).  It does so for bf16 layers
 * with G*C % 256 == 0, H % 256 == 0, M % 32 == 0 and M >= 128; other shapes run the
 * dispatch kernel.  The results are bit-identical either way.
 * Pure host function: *fused = 1 or 0; returns MOE_OK or the config's error.
 */
int moe_forward_fuses_dispatch(const moe_config* cfg, int* fused);

/*
 * Whether moe_forward (and moe_expert_ffn with fill and ws) multiplies only the occupied
 * expert rows for this config (Section 2.2, "Expert capacity"): the kept rows of an expert
 * are packed to the front of its block of G*C rows and only the ceil(kept / 256) row tiles
 * that hold them go through the two GEMMs.  It does so for bf16 layers with G*C, M and H
 * all multiples of 256.  moe_forward_train keeps every slot in place.
 * Pure host function: *packed = 1 or 0; returns MOE_OK or the config's error.
 */
int moe_forward_packs_rows(const moe_config* cfg, int* packed);

/*
 * moe_forward with stage timing marks, for callers that measure the kernels of
 * Algorithm 2 one by one.  Identical work on the same stream; in addition the
 * caller's MOE_FORWARD_EVENTS events (hipEvent_t handles created with timing
 * enabled; host array of handles) are recorded on `stream`:
 *   [0] start  [1] after gating  [2] after dispatch  [3] after h = relu(buf.wi)
 *   [4] after out = h.wo  [5] after combine.
 * When the dispatch is folded into the first GEMM (moe_forward_fuses_dispatch), [2] is
 * recorded directly after [1].
 * events == NULL is exactly moe_forward.  The events stay owned by the caller.
 */
#define MOE_FORWARD_EVENTS 6
int moe_forward_events(const moe_config* cfg, const void* x, const float* wg, const float* u,
                       const void* wi, const void* wo, void* y, float* aux,
                       void* ws, size_t ws_bytes, void* stream, void* const* events);

/* moe_forward_events with pre-packed gate weights (see moe_gate_pack). */
int moe_forward_prepacked(const moe_config* cfg, const void* x, const float* wg,
                          const void* wg_packed, const float* u, const void* wi, const void* wo,
                          void* y, float* aux, void* ws, size_t ws_bytes, void* stream,
                          void* const* events);

/*
 * ---- Backward pass -------------------------------------------------------------
 * The paper trains the layer by differentiating Algorithm 2 automatically; of the
 * auxiliary loss it states that the counts c_e carry no gradient and the mean gates
 * m_e do (Section 2.2, "Auxiliary loss").  The entry points below compute that
 * derivative by the chain rule.  All discrete decisions of Algorithm 1 (top-2 indices,
 * capacity tests, random routing, c_e) are constants; the normalised weights
 * g1/(g1+g2), g2/(g1+g2) are differentiated with respect to both raw gates; a choice
 * that is not kept contributes nothing; relu'(0) = 0.  With
 *   L = sum dy[g,s,m] y[g,s,m] + sum_g daux[g] l_aux[g]
 * the outputs are dL/dx, dL/dwg, dL/dwi, dL/dwo.
 */

/*
 * moe_forward that also keeps the softmax gates g[G,S,E] (fp32) in the workspace, which
 * the backward pass reads together with the routing tensors, h and out.  Same arguments
 * and results as moe_forward; ws: at least moe_train_workspace_bytes(cfg).
 */
int moe_forward_train(const moe_config* cfg, const void* x, const float* wg, const float* u,
                      const void* wi, const void* wo, void* y, float* aux,
                      void* ws, size_t ws_bytes, void* stream);

/* Bytes of workspace moe_backward needs (its own; the forward workspace comes on top).
 * Pure host function. */
int moe_backward_workspace_bytes(const moe_config* cfg, size_t* bytes);

/*
 * Backward of the whole layer (Eq. 1-3 and Algorithms 1-2 differentiated):
 *   dout[e,g,c,:] = weight[g,s,k] dy[g,s,:],  dweight[g,s,k] = <dy[g,s,:], out[e,g,c,:]>
 *   dh   = (dout . wo^T) where h > 0          dwo[e] = h[e]^T . dout[e]
 *   dbuf = dh . wi^T                          dwi[e] = buf[e]^T . dh[e]
 *   dgate: d(g1/(g1+g2)), d(g2/(g1+g2)) for kept choices, + daux[g] c_e / (E S^2)
 *   dz   = g (dgate - <g, dgate>)             (softmax)
 *   dwg  = sum_tokens x^T dz                  dx = sum_k dbuf[e_k,g,c_k,:] + dz . wg^T
 * in : x, wg, wi, wo as given to the forward call;  dy [G,S,M] act_dtype;
 *      daux [G] fp32 (gradient of the loss with respect to each group's l_aux);
 *      fwd_ws: the workspace that a moe_forward_train call with the same cfg, x, wg, u,
 *      wi, wo has filled (read only here; fwd_ws_bytes >= moe_train_workspace_bytes)
 * out: dx [G,S,M] act_dtype;  dwg [M,E] fp32;  dwi [E,M,H], dwo [E,H,M] act_dtype.
 *      Every output element is written (no accumulation into previous contents).
 * ws : at least moe_backward_workspace_bytes(cfg), 256-byte aligned, overwritten.
 * bf16: operands bf16, accumulation fp32, dout / dh / dbuf rounded to bf16 once each;
 * the gate path (dweight, dz, dwg) is fp32.  Sums over tokens run in a fixed order:
 * results are reproducible bit for bit.
 */
int moe_backward(const moe_config* cfg, const void* x, const float* wg, const void* wi,
                 const void* wo, const void* dy, const float* daux,
                 const void* fwd_ws, size_t fwd_ws_bytes,
                 void* dx, float* dwg, void* dwi, void* dwo,
                 void* ws, size_t ws_bytes, void* stream);

/*
 * moe_backward with stage timing marks (see moe_forward_events): MOE_BACKWARD_EVENTS
 * caller-owned events recorded on `stream`:
 *   [0] start  [1] after dout, dweight  [2] after dh  [3] after dwo  [4] after dbuf
 *   [5] after dwi (includes re-dispatching x)  [6] after dz, dwg  [7] after dx.
 * events == NULL is exactly moe_backward.
 */
#define MOE_BACKWARD_EVENTS 8
int moe_backward_events(const moe_config* cfg, const void* x, const float* wg, const void* wi,
                        const void* wo, const void* dy, const float* daux,
                        const void* fwd_ws, size_t fwd_ws_bytes,
                        void* dx, float* dwg, void* dwi, void* dwo,
                        void* ws, size_t ws_bytes, void* stream, void* const* events);

/*
 * ---- The encoder layers around the MoE layer ---------------------------------------
 * Section 2.1: an encoder layer is a self-attention layer followed by a position-wise
 * feed-forward layer, with residual connections and layer normalisation; the MoE
 * Transformer replaces every other feed-forward layer by the MoE layer.  Model sizes of the
 * paper (Appendix, "Machine Translation Experiments Details"): M = 1024, H = 8192, 16 heads
 * of key/value dimension 128.  The entry points below evaluate (forward) one dense and one
 * MoE encoder layer,
 *     a = x + Attention_1(LN_1(x))      b = a + FFN(LN_2(a))
 *     c = b + Attention_2(LN_3(b))      y = c + MoE(LN_4(c))
 * with: layer normalisation first in every sub-layer (the paper does not fix the order),
 * LN(v) = gamma (v - mean) / sqrt(var + 1e-6) + beta over M (population variance);
 * Attention(u) = concat_h softmax(Q_h K_h^T / sqrt(d)) V_h . wo with [Q|K|V] = u . wqkv,
 * no biases, no mask (all sequences have length L), no dropout; FFN(u) = relu(u w1) w2.
 * Tokens are the rows of a [B, L, M] batch and, unchanged in order, the [G, S, M] tokens of
 * the MoE layer (B*L == G*S).  Element types as everywhere: activations and weight matrices
 * cfg->act_dtype, LN parameters and the gate fp32; fp32 accumulation; every stored
 * intermediate is rounded once.
 */
typedef struct {
  int32_t B, L;      /* sequences and their length; B*L == cfg->G * cfg->S */
  int32_t heads, d;  /* attention heads and key/value dimension; A = heads*d */
} moe_encoder_dims;

typedef struct {       /* device pointers, owned by the caller */
  const float *ln_gamma[4], *ln_beta[4]; /* [M] each, sub-layers in the order of the formulas */
  const void *wqkv[2];                   /* [M, 3A]: columns [0,A) = Wq, [A,2A) = Wk, [2A,3A) = Wv */
  const void *wo_att[2];                 /* [A, M] */
  const void *w1, *w2;                   /* dense feed-forward layer: [M,H], [H,M] */
  const float *wg;                       /* MoE layer, as in moe_forward */
  const void *wi, *wo;
} moe_encoder_weights;

/* s = x + delta (delta may be NULL: then s = x and sum_out is not written) and
 * n = LN(s), rows = G*S.  in: x, delta [G,S,M]; gamma, beta [M] fp32
 * out: sum_out [G,S,M] (NULL allowed when delta is NULL); norm_out [G,S,M]. */
int moe_add_layer_norm(const moe_config* cfg, const void* x, const void* delta,
                       const float* gamma, const float* beta, void* sum_out, void* norm_out,
                       void* stream);

/* Bytes of workspace of moe_self_attention / moe_encoder_pair_forward.  Pure host functions. */
int moe_attention_workspace_bytes(const moe_config* cfg, const moe_encoder_dims* dims, size_t* bytes);
int moe_encoder_workspace_bytes(const moe_config* cfg, const moe_encoder_dims* dims, size_t* bytes);

/* out = Attention(u) (no residual): u [B,L,M], wqkv [M,3A], wo_att [A,M] -> out [B,L,M].
 * The flash-style MFMA kernel serves bf16 with d in {64,128} and L % 128 == 0; other
 * shapes use a plain kernel that needs (L + d) * 16 bytes of LDS <= 64 KB. */
int moe_self_attention(const moe_config* cfg, const moe_encoder_dims* dims, const void* u,
                       const void* wqkv, const void* wo_att, void* out,
                       void* ws, size_t ws_bytes, void* stream);

/* out = relu(u w1) w2: u [G,S,M], w1 [M,H], w2 [H,M]; h_ws [G,S,H] scratch. */
int moe_dense_ffn(const moe_config* cfg, const void* u, const void* w1, const void* w2,
                  void* h_ws, void* out, void* stream);

/* The two encoder layers of the formulas above.  in: x [B,L,M], weights, u [G,S] (uniforms of
 * the MoE layer's random routing).  out: y [B,L,M], aux [G].  ws >= moe_encoder_workspace_bytes,
 * 256-byte aligned.  Exactly the sequence moe_add_layer_norm, moe_self_attention,
 * moe_dense_ffn, moe_forward, with the residual sums in between. */
int moe_encoder_pair_forward(const moe_config* cfg, const moe_encoder_dims* dims, const void* x,
                             const moe_encoder_weights* w, const float* u, void* y, float* aux,
                             void* ws, size_t ws_bytes, void* stream);

/* ---- training of the two encoder layers ----------------------------------------------------
 * The paper trains the model by automatic differentiation (Section 2.1 names the sub-layers,
 * Section 3.1 the MoE layer); these entry points evaluate the derivative of
 *     L = sum dy * y + sum_g daux[g] * aux[g]
 * for the pair of layers above by the chain rule: layer normalisation, the attention
 * projections and the scaled dot-product core (probabilities recomputed from q, k and a stored
 * row statistic), the dense feed-forward layer (relu'(0) = 0) and the MoE layer
 * (moe_backward).  Residual branches add their gradients. */
typedef struct {       /* device pointers to the outputs, owned by the caller; shapes as the weights */
  float *ln_gamma[4], *ln_beta[4];
  void *wqkv[2];
  void *wo_att[2];
  void *w1, *w2;
  float *wg;
  void *wi, *wo;
} moe_encoder_grads;

/* Bytes of workspace of moe_encoder_pair_forward_train / moe_encoder_pair_backward.  Host only. */
int moe_encoder_train_workspace_bytes(const moe_config* cfg, const moe_encoder_dims* dims, size_t* bytes);
int moe_encoder_backward_workspace_bytes(const moe_config* cfg, const moe_encoder_dims* dims, size_t* bytes);

/* moe_encoder_pair_forward with the same result, keeping in ws (>= moe_encoder_train_workspace_bytes,
 * 256-byte aligned) what the backward pass reads: the four normalised inputs, the residual sums,
 * q|k|v, the attention context and its row statistic per layer, the hidden activations of the
 * dense layer and the MoE layer's training workspace.  ws must stay untouched until
 * moe_encoder_pair_backward has run. */
int moe_encoder_pair_forward_train(const moe_config* cfg, const moe_encoder_dims* dims, const void* x,
                                   const moe_encoder_weights* w, const float* u, void* y, float* aux,
                                   void* ws, size_t ws_bytes, void* stream);

/* in: x, w as in the forward call; dy [B,L,M] (activation dtype), daux [G] fp32; fwd_ws as left by
 * moe_encoder_pair_forward_train.  out: dx [B,L,M]; every member of g (fully overwritten).
 * ws >= moe_encoder_backward_workspace_bytes, 256-byte aligned.  Errors as the other calls;
 * MOE_EUNSUPPORTED also when the attention shape is served by neither form of the core's
 * derivative: the MFMA kernels take bf16 with d in {64,128} and L % 128 == 0, the plain kernels
 * need (2 L + 2 d) * 16 bytes of LDS <= 64 KB; and when M * 16 bytes > 64 KB (layer-norm
 * parameter sums).  Results are bit-reproducible (no atomics). */
int moe_encoder_pair_backward(const moe_config* cfg, const moe_encoder_dims* dims, const void* x,
                              const moe_encoder_weights* w, const void* dy, const float* daux,
                              const void* fwd_ws, size_t fwd_ws_bytes, void* dx,
                              const moe_encoder_grads* g, void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_GFX950_H */
