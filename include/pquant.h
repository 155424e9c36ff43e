/* libpquant — the pQuant decoupled linear layer on MI355X (gfx950), C ABI.
 *
 * The layer (paper Sec. 3.1-3.3):
 *     Y = beta * (lambda / gamma_t) * Sign(W - mu) * Q(x_t)  +  alpha * HP(x_t)
 * with mu = mean(W), lambda = mean(|W|) per tensor, Q the per-token AbsMax INT8 quantiser
 * (gamma_t = 128 / max_k |x_tk|, round half to even, clamp to [-128, 127]), alpha/beta the
 * learnable feature scales, and HP a compact 16-bit branch: absent, one low-rank pair B(Ax), or
 * E routed experts selected by a linear softmax router with top-k gating.
 *
 * Conventions for every call
 *   - Every pointer is a DEVICE pointer owned by the caller unless marked "host".  The library
 *     never allocates, frees or keeps a pointer after the call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is enqueued on
 *     it and the call returns without waiting.
 *   - Matrices are row-major.  W is [d_out][d_in] (Y = W x).  16-bit tensors are bfloat16.
 *   - Device buffers must be 16-byte aligned; d_in must be a multiple of 32; the training calls
 *     also need d_out % 32 == 0 and hp_rank % 8 == 0.
 *   - Return value: PQ_OK (0) or a negative pq_status.  Nothing throws or aborts;
 *     pq_last_error_string() gives the calling thread's last message.  Arguments are validated on
 *     the host before any kernel is launched, so a call refused for its arguments has enqueued nothing; a
 *     PQ_ERR_HIP from a launch in the middle of a call's sequence leaves the earlier kernels of that call enqueued.
 */
#ifndef PQUANT_H
#define PQUANT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum pq_status {
  PQ_OK = 0,
  PQ_ERR_BAD_ARG = -1,   /* NULL where a buffer is required, negative size, unknown enum */
  PQ_ERR_SHAPE = -2,     /* alignment / divisibility rule violated */
  PQ_ERR_DTYPE = -3,     /* dtype not supported by this call */
  PQ_ERR_WORKSPACE = -4, /* ctx or workspace smaller than pq_*_bytes() says */
  PQ_ERR_HIP = -5        /* a HIP runtime call or kernel launch failed */
} pq_status;

typedef enum pq_dtype { PQ_F32 = 0, PQ_BF16 = 1 } pq_dtype;
typedef enum pq_w_kind { PQ_W_MASTER = 0, PQ_W_PACKED = 1 } pq_w_kind;
typedef enum pq_ste_mode { PQ_STE_IDENTITY = 0, PQ_STE_CLIP = 1 } pq_ste_mode;
/* Form of the high-precision branch (used when hp_rank > 0): 16-bit weights on the unquantised x (the FP16 variant of
 * Sec. 4.6), or the INT8 form of Sec. 3.2 (8-bit weights quantised like the 8-bit activations; see pq_hp_int8_fwd). */
typedef enum pq_hp_kind { PQ_HP_LOWRANK_BF16 = 0, PQ_HP_LOWRANK_INT8 = 1 } pq_hp_kind;

/* One decoupled linear.  Plain data, passed by pointer (host memory). */
typedef struct pq_linear_desc {
  int32_t tokens;    /* T */
  int32_t d_in;      /* K, multiple of 32 */
  int32_t d_out;     /* N */
  int32_t hp_rank;   /* r per expert; 0 = pure 1-bit linear (the attention projections, Sec. 3.1) */
  int32_t n_experts; /* E >= 1; E == 1 is the single dense branch of Sec. 3.2 (no router) */
  int32_t top_k;     /* experts per token, 1 <= top_k <= E (Sec. 3.3 uses 1; Sec. 4.6 tries 2) */
  int32_t io_dtype;  /* pq_dtype of X, Y, dY, dX, the hp weights and the router weights */
  int32_t w_kind;    /* PQ_W_MASTER: latent W given, binarised in the call; PQ_W_PACKED: bits given */
  int32_t ste_mode;  /* PQ_STE_IDENTITY (the paper's STE) or PQ_STE_CLIP: dW *= 1[|W - mu| <= tau] */
  float ste_tau;
  float alpha;       /* scale of the high-precision branch (Sec. 3.2) */
  float beta;        /* scale of the 1-bit branch (Sec. 3.2) */
  int32_t hp_kind;   /* pq_hp_kind; PQ_HP_LOWRANK_INT8 needs n_experts == 1, bf16 I/O, d_out and hp_rank multiples of 32 */
} pq_linear_desc;

int pq_version(void);
const char* pq_last_error_string(void); /* host string, valid until the thread's next failing call */

/* AbsMax INT8 activation quantiser (Sec. 3.1): per token t, gamma_t = 128 / max(max_k |x_tk|, 1e-5)
 * (IEEE fp32 division), q = clamp(rne(fl32(x * gamma_t)), -128, 127).
 *   X [T][K] of `dtype`; Xq [T][K] int8 out; gamma [T] fp32 out.  K % 32 == 0. */
int pq_quant_act(const void* X, int32_t dtype, int32_t T, int32_t K, int8_t* Xq, float* gamma,
                 void* stream);

/* RMSNorm fused with the activation quantiser (Sec. 3.1: Y = (lambda/gamma) W Q(Norm(X)); App. A: the
 * normalisation and the quantiser are both element-wise per token and merge; App. B: RMSNorm).  Per token t:
 *     rstd_t = (mean_k x_tk^2 + eps)^(-1/2)   (mean and rstd in fp64, rstd rounded once to fp32),
 *     xhat_tk = fl32(fl32(x_tk * rstd_t) * g_k), rounded to `dtype` (the stored normalised activation),
 *     gamma_t, q_tk = the quantiser of pq_quant_act applied to the stored xhat.
 *   X [T][K], gain [K] of `dtype`;  Xq [T][K] int8 out, gamma [T] fp32 out;
 *   Xn [T][K] of `dtype` out or NULL (xhat: input of the high-precision branch and of the backward);
 *   Xt [T][K] bf16 out or NULL (q / gamma, what the STE weight gradient multiplies with);
 *   rstd [T] fp32 out or NULL.
 * K % 32 == 0 and K <= 8192 (bf16) / 4096 (fp32): a token's row is read from memory once. */
int pq_rmsnorm_quant_fwd(const void* X, const void* gain, int32_t dtype, int32_t T, int32_t K, float eps, void* Xn,
                         int8_t* Xq, float* gamma, void* Xt, float* rstd, void* stream);
/* Backward of the normalisation for an upstream gradient dXn with respect to xhat (the quantiser itself is
 * differentiated as identity, App. B.1).  With u = x * rstd:
 *     dX_tk = rstd_t * (g_k dXn_tk - u_tk * mean_j(g_j dXn_tj u_tj)),    dgain_k = sum_t dXn_tk u_tk.
 *   dXn, X [T][K], gain [K] of `dtype`; rstd [T] fp32 as written by the forward; dX [T][K] of `dtype` out;
 *   dgain [K] fp32 out (two-stage reduction in a fixed order).  K <= 4096 (bf16) / 2048 (fp32).
 * workspace: at least pq_rmsnorm_bwd_workspace_bytes(T, K) bytes of scratch. */
size_t pq_rmsnorm_bwd_workspace_bytes(int32_t T, int32_t K);
int pq_rmsnorm_bwd(const void* dXn, const void* X, const void* gain, const float* rstd, int32_t dtype, int32_t T,
                   int32_t K, void* dX, float* dgain, void* workspace, size_t workspace_bytes, void* stream);

/* pq_rmsnorm_bwd for callers that cannot allocate or bring a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arguments, results bit-identical to pq_rmsnorm_bwd, but
 * the partial rows of dgain live in a device array that is part of the library image (each GPU the library runs
 * on holds pq_rmsnorm_bwd_static_max_bytes() = 4 MiB of it until the process ends).  The call allocates nothing.
 * Limit: ceil(T / 16) * K * 4 bytes must not exceed that size (e.g. T = 8192 at K = 2048), else
 * PQ_ERR_WORKSPACE and nothing is launched.  Every call on a GPU uses that GPU's one array: calls that overlap
 * on one GPU (two streams, two threads) race; calls on one stream are ordered.  Nothing needs clearing between
 * calls: a call overwrites every partial row it later reads. */
size_t pq_rmsnorm_bwd_static_max_bytes(void);
int pq_rmsnorm_bwd_static(const void* dXn, const void* X, const void* gain, const float* rstd, int32_t dtype, int32_t T,
                          int32_t K, void* dX, float* dgain, void* stream);

/* Weight statistics + binariser + packer (Sec. 3.1 eqs. for W^INT1, mu, lambda; App. A packing).
 * mu and lambda are fp64 sums divided in fp64 and rounded once to fp32; bit = [W >= mu] (so W == mu
 * maps to +1).  packed [N][ceil(K/32)] uint32: bit j of word w <-> column 32 w + j, 1 <-> +1 (the same byte
 * stream as 8 weights per byte, LSB first).  packed_t, if not NULL, receives the transposed packing
 * [K][ceil(N/32)] (bit j of word w <-> row 32 w + j).  mu_lambda [2] fp32 out.
 * K must be a multiple of 4 and N*K of 8.  Widths that are not whole words (Table 1: D_ff - r = 5076 for the 1.3B
 * model) are padded: bits beyond column K - 1 (row N - 1 in packed_t) are 1 (+1); they take no part in mu or
 * lambda and only ever meet an activation code of zero.
 * workspace: at least pq_pack_workspace_bytes(N, K) bytes of scratch. */
size_t pq_pack_workspace_bytes(int32_t N, int32_t K);
int pq_pack_sign(const void* W, int32_t w_dtype, int32_t N, int32_t K, uint32_t* packed,
                 uint32_t* packed_t, float* mu_lambda, void* workspace, size_t workspace_bytes,
                 void* stream);

/* Router (Sec. 3.3): logits = X Wr^T accumulated in fp64 and rounded once to fp32; the k largest
 * logits per token in descending order, ties to the lower expert index; gate = softmax(logits)
 * over all E experts at the selected indices (not renormalised).
 *   X [T][K], Wr [E][K] of `dtype`; idx [T][k] int32, gate [T][k] fp32, probs [T][E] fp32 or NULL.
 *   E <= 64. */
int pq_router_topk(const void* X, const void* Wr, int32_t dtype, int32_t T, int32_t K, int32_t E,
                   int32_t k, int32_t* idx, float* gate, float* probs, void* stream);

/* Integer accumulator of the 1-bit branch, acc[t][n] = sum_k Xq[t][k] * S[n][k] with S read from
 * packed bits (Sec. 3.1, the W1A8 product).  Exact int32.  For tests and tools; pq_linear_fwd
 * runs the same kernel with the de-quantising epilogue.  acc [T][N] int32 out; N % 8 == 0. */
int pq_onebit_acc(const int8_t* Xq, const uint32_t* packed, int32_t T, int32_t K, int32_t N,
                  int32_t* acc, void* stream);

/* Sizes of the caller-owned buffers of pq_linear_fwd / pq_linear_bwd for a descriptor.
 * ctx holds what forward saves for backward (packed bits in both orientations, mu/lambda, the
 * quantised activations and gamma, the hp hidden state, routing decisions); workspace is scratch
 * whose contents need not survive between calls.  Both sizes cover forward and backward. */
size_t pq_linear_ctx_bytes(const pq_linear_desc* desc);
size_t pq_linear_workspace_bytes(const pq_linear_desc* desc);

/* Forward of the decoupled linear (Sec. 3.1 last eq., Sec. 3.2 FFN eq., Sec. 3.3).
 *   X [T][K] io_dtype.
 *   W_or_packed: PQ_W_MASTER -> latent W [N][K] io_dtype; PQ_W_PACKED -> uint32 [N][K/32].
 *   mu_lambda [2] fp32: read when PQ_W_PACKED; ignored (may be NULL) when PQ_W_MASTER, where the
 *     statistics are computed and stored in ctx.
 *   hpA: E == 1: [r][K]; E > 1: [E][r][K].   hpB: E == 1: [N][r]; E > 1: [E][N][r].  io_dtype.
 *   Wr [E][K] io_dtype, only for E > 1.  All three NULL when hp_rank == 0.
 *   E > 1 (Sec. 3.3; bf16 I/O only, d_out % 32 == 0): the router of pq_router_topk selects top_k experts per token,
 *   the tokens are permuted by expert (stable), H_e = X_e A_e^T and Y_e = H_e B_e^T run as grouped GEMMs over the
 *   expert segments (both stored in bf16), and Y += alpha * sum_j gate_j Y_e_j in token order.
 *   hp_kind == PQ_HP_LOWRANK_INT8 (E == 1): the branch of pq_hp_int8_fwd on the codes the 1-bit branch has just
 *   formed (x is quantised once), added to the 1-bit branch's rounded output.
 *   Y [T][N] io_dtype out.
 *   ctx: pq_linear_ctx_bytes() bytes, or NULL for inference (nothing saved; no backward).
 *   workspace: pq_linear_workspace_bytes() bytes. */
int pq_linear_fwd(const pq_linear_desc* desc, const void* X, const void* W_or_packed,
                  const float* mu_lambda, const void* hpA, const void* hpB, const void* Wr, void* Y,
                  void* ctx, size_t ctx_bytes, void* workspace, size_t workspace_bytes, void* stream);

/* STE backward (Sec. 4 intro, App. B.1): Sign and Q are differentiated as identity; mu, lambda and
 * gamma carry no gradient.
 *   dY [T][N] io_dtype; X, W, hpA, hpB, Wr as given to forward; ctx as written by forward.
 *   dX [T][K] io_dtype out.  dW [N][K] fp32 out (gradient of the latent weight).
 *   dhpA, dhpB, dWr: fp32 out, shaped like hpA, hpB, Wr (NULL when that input is absent).  For E > 1 the router's
 *   softmax gate is differentiated too: dgate = alpha <dY_t, Y_e(x_t)>, dWr and its part of dX follow.
 *   dalpha_dbeta [2] fp32 out: {dL/dalpha, dL/dbeta}.
 * Reductions are two-stage with a fixed order: results are bit-identical from run to run. */
int pq_linear_bwd(const pq_linear_desc* desc, const void* dY, const void* X, const void* W,
                  const void* hpA, const void* hpB, const void* Wr, const void* ctx, size_t ctx_bytes,
                  void* dX, float* dW, float* dhpA, float* dhpB, float* dWr, float* dalpha_dbeta,
                  void* workspace, size_t workspace_bytes, void* stream);

/* The decoupled linear with its normalisation in front (Sec. 3.1 prints Y = (lambda/gamma) W Q(Norm(X)); App. B
 * names RMSNorm): pq_linear_fwd / pq_linear_bwd applied to xhat = RMSNorm(X) * gain, with the normalisation fused
 * into the activation quantiser (pq_rmsnorm_quant_fwd writes the codes into ctx; X is read from memory once) and the
 * normalisation backward (pq_rmsnorm_bwd) chained behind the linear's dX.  The high-precision branch reads xhat.
 *   X [T][K], gain [K] io_dtype; eps >= 0; W latent weights (PQ_W_MASTER); the other arguments as in pq_linear_fwd.
 *   Backward: dX [T][K] io_dtype is the gradient with respect to X; dgain [K] fp32.
 *   ctx / workspace: pq_linear_norm_ctx_bytes() / pq_linear_norm_workspace_bytes() bytes (ctx is required).
 *   d_in <= 8192 (bf16) / 4096 (fp32) for the forward, 4096 / 2048 for the backward. */
size_t pq_linear_norm_ctx_bytes(const pq_linear_desc* desc);
size_t pq_linear_norm_workspace_bytes(const pq_linear_desc* desc);
int pq_linear_norm_fwd(const pq_linear_desc* desc, const void* X, const void* gain, float eps, const void* W,
                       const void* hpA, const void* hpB, const void* Wr, void* Y, void* ctx, size_t ctx_bytes,
                       void* workspace, size_t workspace_bytes, void* stream);
int pq_linear_norm_bwd(const pq_linear_desc* desc, const void* dY, const void* X, const void* gain, const void* W,
                       const void* hpA, const void* hpB, const void* Wr, const void* ctx, size_t ctx_bytes, void* dX,
                       float* dgain, float* dW, float* dhpA, float* dhpB, float* dWr, float* dalpha_dbeta,
                       void* workspace, size_t workspace_bytes, void* stream);

/* INT8 form of the two-factor high-precision branch (Sec. 3.2: the 8-bit weights are quantised identically to
 * the 8-bit activations; Sec. 3.1 quantiser).  With Q the AbsMax INT8 quantiser of pq_quant_act applied per row:
 *     (q_a, g_a) = Q(A),  (q_b, g_b) = Q(B),   acc1 = q_x q_a^T (exact int32),
 *     H = fl32(fl32(fl32(1/g_x[t]) * fl32(acc1)) / g_a[j]) rounded to bf16,  (q_h, g_h) = Q(H),
 *     acc2 = q_h q_b^T (exact int32),   Y (+)= fl32(fl32(fl32(alpha/g_h[t]) * fl32(acc2)) / g_b[n]).
 *   Xq [T][K] int8 and gamma_x [T] fp32: codes of X as written by pq_quant_act / pq_rmsnorm_quant_fwd (the 1-bit
 *   branch's own, nothing is quantised twice);  A [r][K], B [N][r] bf16;  Y [T][N] bf16, overwritten or, with
 *   accumulate != 0, added to (the 1-bit branch's output).  ctx receives what the backward needs.
 * Backward (STE, App. B.1: every quantiser is the identity): with X~ = q_x/g_x (Xt [T][K] bf16 as written by the
 * quantiser), A~, B~, H~ likewise:  dH = alpha dY B~,  dB = alpha dY^T H~,  dA = dH^T X~,  dX (+)= dH A~.
 *   dY [T][N] bf16;  dX [T][K] bf16 (overwritten, or added to with accumulate_dX != 0);  dA [r][K], dB [N][r] fp32.
 * bf16 only; K, N and r multiples of 32.  ctx / workspace sizes from the two queries. */
size_t pq_hp_int8_ctx_bytes(int32_t T, int32_t K, int32_t N, int32_t r);
size_t pq_hp_int8_workspace_bytes(int32_t T, int32_t K, int32_t N, int32_t r);
int pq_hp_int8_fwd(const int8_t* Xq, const float* gamma_x, const void* A, const void* B, int32_t dtype, int32_t T,
                   int32_t K, int32_t N, int32_t r, float alpha, void* Y, int32_t accumulate, void* ctx,
                   size_t ctx_bytes, void* workspace, size_t workspace_bytes, void* stream);
int pq_hp_int8_bwd(const void* dY, const void* Xt, int32_t dtype, int32_t T, int32_t K, int32_t N, int32_t r,
                   float alpha, const void* ctx, size_t ctx_bytes, void* dX, int32_t accumulate_dX, float* dA, float* dB,
                   void* workspace, size_t workspace_bytes, void* stream);

/* Group-wise scales of the 1-bit weights, the variant Sec. 4.6 evaluates against the per-tensor scale and rejects
 * (one 16-bit scale per 64 one-bit weights: metadata overhead, unfriendly to hardware).  Built as a measured contrast,
 * forward only:
 *     group = 64:  Y[t][n] = beta / gamma_t * sum_g lambda[n][g] * sum_{k in group g} S[n][k] q[t][k],
 *                  lambda[n][g] = mean |W[n][64 g .. 64 g + 63]| rounded to fp32 and then to fp16;
 *     group = 0:   the per-tensor product of Sec. 3.1, Y[t][n] = beta * lambda / gamma_t * sum_k S[n][k] q[t][k], in the
 *                  same kernel (int32 accumulation over the whole contraction), so that the two timings differ by the
 *                  group scales alone.
 * mu, S = Sign(W - mu), q and gamma are those of pq_linear_fwd (Sec. 3.1).
 *   X [T][K], W [N][K] bf16 (dtype must be PQ_BF16);  Y [T][N] fp32, overwritten;  K % 64 == 0, N % 32 == 0.
 *   workspace: device memory of pq_groupwise_workspace_bytes(T, K, N) bytes (codes, scales, packed signs, group scales);
 *   the caller keeps ownership of every buffer.  Errors as everywhere: a negative pq_status, message via pq_last_error. */
size_t pq_groupwise_workspace_bytes(int32_t T, int32_t K, int32_t N);
int pq_groupwise_fwd(const void* X, const void* W, int32_t dtype, int32_t T, int32_t K, int32_t N, int32_t group, float beta,
                     float* Y, void* workspace, size_t workspace_bytes, void* stream);

/* The decoupled FFN (Sec. 3.2 FFN equation; Sec. 3.3):
 *     Y = beta * FFN_1bit(X) + alpha * sum_j gate_j(X) * FFN_e_j(X)
 * FFN_1bit: U = L_up(Q(X)), G = L_gate(Q(X)) (pure 1-bit linears, Sec. 3.1), Hd = silu(G) * U,
 * Y1 = L_down(Q(Hd)); U and G are stored in bf16, Hd is formed in fp32 and re-quantised per token.
 * FFN_e: gated bf16 expert of hidden width r, Down_e (silu(Gate_e x) * Up_e x); the router of
 * pq_router_topk picks top_k experts per token; tokens are permuted by expert (stable), the experts
 * run as grouped GEMMs and the results are combined in token order.
 *   X [T][d] bf16;  W_up, W_gate [F][d], W_down [d][F] bf16 latent weights;
 *   Up, Gate [E][r][d], Down [E][d][r], Wr [E][d] bf16;  Y [T][d] bf16 out.
 *   Backward (STE as in pq_linear_bwd): dX [T][d] bf16; dW_up, dW_gate [F][d], dW_down [d][F], dUp,
 *   dGate [E][r][d], dDown [E][d][r], dWr [E][d] fp32; dalpha_dbeta [2] fp32.
 * hp_kind == PQ_HP_LOWRANK_INT8 (Sec. 3.2, FFN^INT8: the 8-bit weights are quantised like the 8-bit activations): the
 * rows of Up_e, Gate_e [r][d] and Down_e [d][r] go through the quantiser of pq_quant_act; an expert reads the codes and
 * gamma of x that the 1-bit branch formed, u = (q_x q_up^T) / (gamma_x gamma_up) and g likewise are stored in bf16,
 * a = silu(g) * u is stored in bf16 and quantised again per token, and the expert's output is (q_a q_down^T) /
 * (gamma_a gamma_down); both products are exact int32 and the scales come off as in pq_hp_int8_fwd.  The backward is
 * the STE one on the de-quantised factors (X~ = q_x / gamma_x, Up~, Gate~, Down~, a~); the router reads x itself.
 * bf16 I/O only; d a multiple of 32, F a multiple of 4, r a multiple of 8, E <= 64.  An F that is not a multiple of 32
 * (Table 1: D_ff - r = 5076 for the 1.3B model) is padded to whole packed words inside the library: the padded hidden
 * units carry zero codes and zero gradients and take no part in mu, lambda or any sum; the caller's tensors keep F. */
typedef struct pq_ffn_desc {
  int32_t tokens, d_model, d_ffn, hp_rank, n_experts, top_k, io_dtype;
  float alpha, beta;
  int32_t hp_kind; /* pq_hp_kind of the experts: PQ_HP_LOWRANK_BF16 (16-bit weights on the unquantised x) or
                      PQ_HP_LOWRANK_INT8 (the form the FFN equation of Sec. 3.2 prints; needs hp_rank % 32 == 0) */
} pq_ffn_desc;
size_t pq_ffn_ctx_bytes(const pq_ffn_desc* desc);
size_t pq_ffn_workspace_bytes(const pq_ffn_desc* desc);
/* Where pq_ffn_fwd leaves the intermediate results it stores in ctx (byte offset and size of a section; rows of U, G and
 * Hq are d_ffn rounded up to a multiple of 32 long): the codes and gammas of x (Sec. 3.1 quantiser), U and G (bf16), the
 * codes and gammas of the gated hidden state Hd.  For inspection; the layout is otherwise the library's own. */
typedef enum pq_ffn_ctx_section_id {
  PQ_FFN_CTX_XQ = 0, PQ_FFN_CTX_GAMMA_X = 1, PQ_FFN_CTX_U = 2, PQ_FFN_CTX_G = 3, PQ_FFN_CTX_HQ = 4, PQ_FFN_CTX_GAMMA_H = 5
} pq_ffn_ctx_section_id;
int pq_ffn_ctx_section(const pq_ffn_desc* desc, int32_t section, size_t* offset, size_t* bytes);
int pq_ffn_fwd(const pq_ffn_desc* desc, const void* X, const void* W_up, const void* W_gate, const void* W_down,
               const void* Up, const void* Gate, const void* Down, const void* Wr, void* Y, void* ctx,
               size_t ctx_bytes, void* workspace, size_t workspace_bytes, void* stream);
int pq_ffn_bwd(const pq_ffn_desc* desc, const void* dY, const void* X, const void* Up, const void* Gate,
               const void* Down, const void* Wr, const void* ctx, size_t ctx_bytes, void* dX, float* dW_up,
               float* dW_gate, float* dW_down, float* dUp, float* dGate, float* dDown, float* dWr,
               float* dalpha_dbeta, void* workspace, size_t workspace_bytes, void* stream);

/* Inference on packed weights for small token batches (App. A): the decode product
 *     y[l][b][n] = (s_l / gamma_lb) * sum_k q[l][b][k] * S_l[n][k]
 *                  + alpha * sum_j gate[l][b][j] * B_le (A_le x_lb),   e = idx[l][b][j]
 * for n_layers independent weight sets l in one launch (n_layers = 1 is a single layer).
 * Everything runs in the call: AbsMax INT8 quantisation of x (Sec. 3.1), router top-k (Sec. 3.3),
 * the expert hidden state, the packed-bit product with exact int32 accumulation, the experts.
 *   X [L][B][K] bf16;  packed [L][N][K/32] uint32 (layout of pq_pack_sign);
 *   scale_fp16 [L]: the bits of fp16(beta * lambda), the single stored scale of a packed layer;
 *   hpA [L][E][r][K], hpB [L][E][N][r], Wr [L][E][K] bf16 (all NULL when hp_rank == 0);
 *   Y [L][B][N] bf16 out;  acc_out [L][B][N] int32 out or NULL (the exact accumulators, for tests).
 * Limits: 1 <= B <= 16; K % 128 == 0 (K % 512 == 0 for B > 1 on the row-major packing); N % 4 == 0;
 * r % 8 == 0 (B == 1) or r % 32 == 0 and (E r) % 64 == 0 (B > 1); for B > 1 the codes and expert
 * hidden states of 8 (B <= 8) or 16 token rows must fit the LDS: rows * (K + 2 E r) <= 160 KiB
 * (row-interleaved packing: the codes pass through in blocks, min(rows * K, 32 KiB) + max(8 KiB, 2 rows E r)).
 * Violations return PQ_ERR_SHAPE. */
typedef enum pq_packed_layout {
  PQ_PACKED_ROWMAJOR = 0, /* [N][K/32], as written by pq_pack_sign */
  PQ_PACKED_TILED64 = 1   /* [ceil(N/64)][K/128][64][4]: rows interleaved by 64 (pq_pack_retile64); any batch, the fast layout */
} pq_packed_layout;
typedef struct pq_decode_desc {
  int32_t batch;     /* B, tokens per layer */
  int32_t d_in;      /* K */
  int32_t d_out;     /* N */
  int32_t hp_rank;   /* r per expert, 0 = no high-precision branch */
  int32_t n_experts; /* E */
  int32_t top_k;     /* experts per token */
  int32_t n_layers;  /* L */
  int32_t packed_layout; /* pq_packed_layout of `packed` */
  float alpha;
} pq_decode_desc;
size_t pq_decode_workspace_bytes(const pq_decode_desc* desc);
/* Offline re-tiling for decode: packed [N][K/32] -> tiled, pq_pack_tiled64_bytes(N, K) bytes, word
 * (row, w) stored at (((row/64) * (K/128) + w/4) * 64 + row%64) * 4 + w%4, rows padded with zeros to a
 * multiple of 64.  In this order a wavefront reads 1 KiB of contiguous memory per load and a group of
 * 64 rows is one contiguous run of 8 K bytes.  K % 128 == 0. */
size_t pq_pack_tiled64_bytes(int32_t N, int32_t K);
int pq_pack_retile64(const uint32_t* packed, int32_t N, int32_t K, uint32_t* tiled, void* stream);
int pq_decode_gemv(const pq_decode_desc* desc, const void* X, const uint32_t* packed, const uint16_t* scale_fp16,
                   const void* hpA, const void* hpB, const void* Wr, void* Y, int32_t* acc_out, void* workspace,
                   size_t workspace_bytes, void* stream);

/* pq_decode_gemv with the routed experts in their INT8 form (Sec. 3.2: the 8-bit weights are quantised like the
 * 8-bit activations; Sec. 3.3; App. A).  Offline, every row of A_le and B_le goes through pq_quant_act:
 *   hpA_q [L][E][r][K] int8 with gamma_A [L][E][r],  hpB_q [L][E][N][r] int8 with gamma_B [L][E][N].
 * Per token and selected expert e (q, gamma_x: the token's codes of the 1-bit branch; the router reads x itself):
 *     H_i  = bf16(fl32(fl32(1/gamma_x) * sum_k q_k A_q[e][i][k]) / gamma_A[e][i]),   (q_h, gamma_h) = Q(H),
 *     Y_en = fl32(fl32(1/gamma_h) * sum_i q_h,i B_q[e][n][i]) / gamma_B[e][n],
 * both sums exact int32, and y = 1-bit product + alpha * sum_j gate_j Y_e_j as in pq_decode_gemv.  The expert
 * weights are read as 1 byte per entry instead of 2.  The workspace is that of pq_decode_gemv; after the call
 * its hidden-state section holds H ([L][top_k][r] fp32 values of the bf16 roundings, for tests).
 * Limits: r % 32 == 0.  batch == 1: top_k <= 8 and top_k * r <= 2048; K % 128 == 0 and K <= 13056.
 * batch > 1: row-interleaved packing only, r % 64 == 0 and (E r) % 128 == 0, otherwise the limits of pq_decode_gemv;
 * there the division by gamma_B is a multiplication by the hardware reciprocal (within 1 ulp of the formula above; H,
 * its codes and both integer sums are unaffected). */
int pq_decode_gemv_int8(const pq_decode_desc* desc, const void* X, const uint32_t* packed, const uint16_t* scale_fp16,
                        const int8_t* hpA_q, const float* gamma_A, const int8_t* hpB_q, const float* gamma_B,
                        const void* Wr, void* Y, int32_t* acc_out, void* workspace, size_t workspace_bytes,
                        void* stream);

/* The decoupled FFN at inference on packed weights, one token per layer (Sec. 3.2 FFN equation, Sec. 3.3,
 * App. A: every scalar of a layer folded into one stored scale), for n_layers independent FFNs per call:
 *     q, gamma = Q(x);  U = bf16((s_up/gamma) S_up q),  G = bf16((s_gate/gamma) S_gate q)   (x quantised once),
 *     Hd = silu(G) * U (fp32),  q_h, gamma_h = Q(Hd),  Y1 = (s_down/gamma_h) S_down q_h,
 *     Y = Y1 + alpha * sum_j gate_j Down_e (silu(Gate_e x) * (Up_e x)),  e = idx_j  (router and experts read x itself).
 *   X [L][D] bf16;  packed_upgate [L][2]: the row-interleaved packing (pq_pack_retile64) of W_up then W_gate,
 *   each pq_pack_tiled64_bytes(F, D) bytes;  scale_upgate [L][2]: fp16 bits of lambda_up, lambda_gate;
 *   packed_down [L]: row-interleaved packing of W_down (pq_pack_tiled64_bytes(D, F) each);  scale_down [L]:
 *   fp16 bits of beta * lambda_down;  UpGate [L][E][2r][D] bf16: the rows of Up_e followed by those of Gate_e;
 *   Down [L][E][D][r], Wr [L][E][D] bf16;  Y [L][D] bf16 out;  acc_upgate [L][2][F] int32 out or NULL (the exact
 *   accumulators of the up and gate products, for tests).
 * Four launches: quantiser + router + expert hidden pairs; the 2 L up/gate products; gated unit + quantiser of
 * Hd; the L down products with the experts' down projections.
 * Limits: D % 128 == 0, F % 128 == 0, both <= 16384; r % 8 == 0, r > 0; 1 <= top_k <= E <= 64.
 * batch = B > 1 (small-batch decoding, App. A): B tokens per layer through the same stages on the small-batch kernels;
 *   X and Y are [L][B][D], acc_upgate [L][2][B][F]; the up and gate products of a layer read the layer's B quantised
 *   tokens once per workgroup, every expert selected by some token is read once per output tile.
 *   Further limits: B <= 16, r % 32 == 0, (E r) % 64 == 0, and the expert hidden states of 8 (B <= 8) or 16 token rows
 *   (2 * rows * E * r bytes, at least 8 KiB) must fit 160 KiB of LDS next to a 32 KiB block of codes. */
typedef struct pq_decode_ffn_desc {
  int32_t d_model;   /* D */
  int32_t d_ffn;     /* F */
  int32_t hp_rank;   /* r: hidden width of an expert */
  int32_t n_experts; /* E */
  int32_t top_k;
  int32_t n_layers;  /* L */
  float alpha;
  int32_t batch;     /* B: tokens per layer, 1..16 (0 stands for 1) */
} pq_decode_ffn_desc;
size_t pq_decode_ffn_workspace_bytes(const pq_decode_ffn_desc* desc);
int pq_decode_ffn(const pq_decode_ffn_desc* desc, const void* X, const uint32_t* packed_upgate, const uint16_t* scale_upgate,
                  const uint32_t* packed_down, const uint16_t* scale_down, const void* UpGate, const void* Down,
                  const void* Wr, void* Y, int32_t* acc_upgate, void* workspace, size_t workspace_bytes, void* stream);

/* Glue for chaining the linears into a layer stack; not part of the method.
 * pq_glue_lincomb: out = c0 x0 + c1 x1 + c2 x2 + c3 x3 over n bf16 elements (x1..x3 may be NULL;
 * fp32 arithmetic, one rounding; n % 8 == 0) -- residual adds and the mean that stands in for the
 * attention core.  pq_glue_gather_rows: out[t][:] = table[ids[t]][:] (bf16 rows of d elements). */
int pq_glue_lincomb(void* out, const void* x0, const void* x1, const void* x2, const void* x3, float c0,
                    float c1, float c2, float c3, size_t n, void* stream);
int pq_glue_gather_rows(const void* table, const int32_t* ids, int32_t T, int32_t d, void* out, void* stream);

/* Per-kernel timing for benchmarks.  While enabled, every kernel launch made by the library is
 * bracketed by a pair of HIP events on the caller's stream (events are created on demand, so this
 * mode allocates; it is off by default).  pq_prof_count() = number of kernel labels;
 * pq_prof_label(i) = host string naming label i; pq_prof_read(i, &ms, &launches) waits for the
 * recorded events of label i and returns their summed duration in milliseconds and their count;
 * pq_prof_reset() drops all recorded samples. */
int pq_prof_enable(int on);
int pq_prof_count(void);
const char* pq_prof_label(int label);
int pq_prof_read(int label, double* total_ms, int* launches);
int pq_prof_reset(void);

#ifdef __cplusplus
}
#endif
#endif /* PQUANT_H */
