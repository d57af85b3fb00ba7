/*
 * zo.h — C ABI of the candidate-state evaluation library for Inference-Native
 * zeroth-order optimisation on AMD MI355X (gfx950).
 *
 * The library evaluates a packed batch of token rows in which every sequence
 * names the candidate state it is scored under (the "ProbePlan" of Sec. 2.2,
 * Eq. 3 of the paper).  A candidate (direction k, sign s) sees
 *
 *     W_c = W_0 + s * eps * U_k V_k^T + P Vb^T            (Sec. 3.2)
 *
 * without W_0 ever being written: the side state is applied as factors
 * (LoRA-style A = V^T, B = +-eps U) next to a persistent low-rank bank
 * (Eq. "bank").  U_k [m x r] and V_k [n x r] are regenerated on the device from
 * a 64-bit seed by a counter-based generator (Philox4x32-10 + Box-Muller) and
 * are never passed across this boundary.  Foreground sequences (candidate id
 * -1) see W_0 alone and their results are bit-identical to a call in which
 * every sequence is foreground (Sec. 5.4 and the mixed-batch correctness appendix).
 *
 * Conventions
 *   - A linear layer has W [m x n] row-major (m = out features, n = in
 *     features); X [T x n] holds packed token rows; Y = X W^T is [T x m].
 *   - Every pointer is a DEVICE pointer unless its name starts with "host_".
 *   - The caller owns every buffer.  Inputs (const) are never written.  Outputs
 *     are fully overwritten.  Scratch memory comes from the caller-provided
 *     `workspace` whose size the *_workspace_bytes queries return (host-only,
 *     pure functions of the shapes).  The library allocates nothing, keeps no
 *     pointer after the work it enqueued has run, and never synchronises.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream); all
 *     device work of a call is enqueued on it, in order.
 *   - Every function returns a zo_status.  All argument validation happens
 *     before the first HIP call, so error paths can be exercised on a machine
 *     without a GPU.  zo_last_error() returns a thread-local message.
 *   - Results are deterministic: no atomics, and reduction orders that are
 *     fixed and do not depend on the batch.  A row's result does not depend
 *     on which other rows share the batch.
 */
#ifndef ZO_H_
#define ZO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum zo_status {
  ZO_OK = 0,
  ZO_ERR_NULL = -1,        /* a required pointer is NULL */
  ZO_ERR_SHAPE = -2,       /* negative size, r outside [1,512], R_used > R_cap, bad leading dimension / alignment */
  ZO_ERR_INDEX = -3,       /* candidate / direction id out of range, malformed cu_seqlens (host mirrors only) */
  ZO_ERR_BANK_FULL = -4,   /* a direction's column block does not fit in the bank */
  ZO_ERR_WORKSPACE = -5,   /* workspace missing, misaligned or too small */
  ZO_ERR_UNSUPPORTED = -6, /* dtype combination or shape the kernels do not cover */
  ZO_ERR_HIP = -7          /* a HIP call failed; zo_last_error() has the HIP string */
} zo_status;

typedef enum zo_dtype { ZO_F32 = 0, ZO_BF16 = 1 } zo_dtype;

/*
 * The packed batch and its candidate table (Sec. 2.2, Eq. 3: each query is a
 * candidate id, an input and an observation; here the input is a sequence of
 * packed rows and the observation is its summed token NLL).
 *
 *   cu_seqlens [S+1]  row offsets, cu[0] = 0, non-decreasing, cu[S] = n_tokens
 *                     (variable-length packing, Sec. 3.1; empty sequences allowed)
 *   seq_cand   [S]    candidate id of each sequence; -1 = foreground (base weights only)
 *   cand_dir   [C]    direction index in [0, n_dirs) of each candidate; -1 = centre
 *                     (bank only, no probe)
 *   cand_sign  [C]    +1, -1 or 0 (0 = centre)
 *   dir_seed   [K]    64-bit seed of each direction; U uses the stream
 *                     (seed, tensor_id & ~1), V the stream (seed, tensor_id | 1)
 *   host_*            optional host copies used only for validation; may be NULL
 *   dir_seed_v [K]    optional (NULL: V is drawn from dir_seed too): separate seeds
 *                     for V, so that one V_k can be reused over an interval of steps
 *                     while U_t is drawn afresh (Sec. 3.2)
 */
typedef struct zo_batch {
  int32_t n_tokens;
  int32_t n_seqs;
  const int32_t* cu_seqlens;
  const int32_t* seq_cand;
  int32_t n_cands;
  const int32_t* cand_dir;
  const float* cand_sign;
  int32_t n_dirs;
  const uint64_t* dir_seed;
  const int32_t* host_cu_seqlens;
  const int32_t* host_seq_cand;
  const int32_t* host_cand_dir;
  const uint64_t* dir_seed_v;
} zo_batch;

/*
 * Persistent update bank of one layer (Sec. 3.2, Eq. "bank"):
 * W_eff = W_0 + P[:, :R_used] Vb[:, :R_used]^T.  fp32 state, row-major,
 * leading dimension R_cap.  P is [m x R_cap], Vb is [n x R_cap].
 */
typedef struct zo_bank {
  int32_t R_cap;
  int32_t R_used;
  float* P;
  float* Vb;
} zo_bank;

/* Library version (major * 1000 + minor). */
int32_t zo_version(void);

/* Copies the calling thread's last error message (NUL-terminated, truncated to
 * cap) into buf; returns the message length. */
size_t zo_last_error(char* buf, size_t cap);

/*
 * Raw words of the factor generator (for parity checks of the integer stream).
 * Block q = first_block + i uses Philox4x32-10 with counter
 * (q mod 2^32, q div 2^32, tensor_id, 0) and key (seed mod 2^32, seed div 2^32).
 * out_words: device uint32 [n_blocks x 4].
 */
int32_t zo_philox_words(uint64_t seed, uint32_t tensor_id, uint64_t first_block,
                        int64_t n_blocks, uint32_t* out_words, void* stream);

/*
 * One factor matrix [rows x r] of i.i.d. standard normals (Sec. 3.3: U and V
 * have independent standard-normal entries).  Entry (i, j) has flat index
 * e = i*r + j and is lane e mod 4 of block e div 4 of the stream
 * (seed, tensor_id): uniforms u(w) = (2 (w >> 9) + 1) 2^-24, lanes (0,1) =
 * sqrt(-2 ln u(w0)) * (cos, sin)(2 pi u(w1)), lanes (2,3) likewise from
 * (w2, w3).  dtype ZO_F32 writes float, ZO_BF16 writes the fp32 value rounded
 * to nearest-even bfloat16.  out: device [rows x r], dense.
 */
int32_t zo_factor_fill(uint64_t seed, uint32_t tensor_id, int64_t rows, int32_t r,
                       zo_dtype dtype, void* out, void* stream);

/*
 * Packing indices of a batch (Sec. 3.1, variable-length packing):
 * tok_seq[t] = the sequence whose row range contains t, tok_cand[t] =
 * seq_cand[tok_seq[t]].  Outputs: device int32 [n_tokens] each (either may be
 * NULL).  Integer results, exact.
 */
int32_t zo_batch_index(const zo_batch* batch, int32_t* tok_seq, int32_t* tok_cand, void* stream);

/*
 * Probe linear (Sec. 3.2, candidate states W_+-, combined probe and bank):
 *
 *   Y[t,:] = act( X[t,:] W^T + s_t eps (X[t,:] V_{k_t}) U_{k_t}^T
 *                 + (X[t,:] Vb) P^T + bias )
 *
 * for rows of candidate sequences; rows of a centre candidate omit the probe
 * term; rows of foreground sequences get act(X W^T + bias) and are
 * bit-identical to an all-foreground call.
 *
 *   X [T x n] ld ldx, W [m x n] ld ldw, Y [T x m] ld ldy  (elements; row-major)
 *   in_dtype  type of X and W and of the factors U, V (ZO_F32: everything fp32
 *             on the vector ALU; ZO_BF16: bf16 operands, fp32 accumulation on
 *             the matrix cores, U and V rounded to bf16)
 *   out_dtype type of Y: equal to in_dtype, or ZO_F32 with ZO_BF16 inputs
 *   bias      fp32 [m] or NULL;  act 0 = none, 1 = ReLU, 2 = gated SiLU (the gated MLP of the
 *             Qwen3 family): output features are (gate_j, up_j) pairs in adjacent rows of W and
 *             Y[t, j] = silu(gate_j) * up_j, silu(x) = x / (1 + exp(-x)); Y then has m/2 columns
 *   r         rank of the probe, 1..512 (the rank continuum of Sec. 3.3; its 1/sqrt(r) goes into eps; the
 *             kernels are laid out for the small ranks of the paper's runs, larger ones cost in proportion);
 *             eps probe scale;  tensor_id even id of the layer
 *   bank      NULL or R_used = 0: no bank
 * ZO_BF16 requires n % 64 == 0 (and, for bf16 output, a multiple of 8 output columns: m % 8 == 0, or
 * m % 16 == 0 with act 2), 16-byte aligned X, W, Y and leading dimensions that keep rows 16-byte aligned.
 * Y [T x m] above means [T x m/2] with act 2.
 */
size_t zo_probe_linear_workspace_bytes(int32_t n_tokens, int32_t n_seqs, int32_t n_dirs,
                                       int32_t m, int32_t n, int32_t r, int32_t R_used,
                                       zo_dtype in_dtype);

int32_t zo_probe_linear(const zo_batch* batch, const void* X, int64_t ldx,
                        const void* W, int64_t ldw, const float* bias,
                        int32_t m, int32_t n, zo_dtype in_dtype,
                        int32_t r, float eps, uint32_t tensor_id,
                        const zo_bank* bank, int32_t act,
                        void* Y, int64_t ldy, zo_dtype out_dtype,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Fused LM-head scoring (Sec. 2.2 token-scoring observation; Sec. 3.3
 * "compact active-token logits or per-request NLL"): logits
 * z_t = H[t,:] W_head^T are never stored;
 *
 *   tok_nll[t]  = log sum_v exp(z_tv) - z_t[targets[t]]   (0 when targets[t] < 0)
 *   seq_nll[s]  = sum of tok_nll over the sequence's rows
 *   cand_sum[c] = sum of seq_nll over sequences with seq_cand == c
 *   cand_cnt[c] = number of scored rows (targets >= 0) of candidate c
 *
 *   H [T x d] ld ldh, W_head [vocab x d] ld ldw (dtype; ZO_BF16 needs d % 64 == 0)
 *   targets int32 [T] in [-inf, vocab)
 *   tok_nll fp32 [T] (nullable), seq_nll fp32 [S], cand_sum fp32 [C], cand_cnt int32 [C]
 * The head carries no side state.  Foreground sequences get seq_nll but
 * contribute to no candidate.  With ZO_BF16 only the rows with a target are
 * multiplied (active-token scoring): the cost of a call follows the number
 * of scored tokens, not T (when H spans less than 2 GiB; a larger H is
 * multiplied whole, with the same results).
 */
size_t zo_score_workspace_bytes(int32_t n_tokens, int32_t n_seqs, int32_t vocab, int32_t d,
                                zo_dtype dtype);

int32_t zo_score(const zo_batch* batch, const void* H, int64_t ldh,
                 const void* W_head, int64_t ldw, int32_t vocab, int32_t d, zo_dtype dtype,
                 const int32_t* targets, float* tok_nll, float* seq_nll,
                 float* cand_sum, int32_t* cand_cnt,
                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * zo_score for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * results and errors as zo_score, without the workspace: the scratch of the scoring
 * kernels (list of scored tokens, per-vocabulary-tile partial maxima and sums,
 * target logits) lives in a static device array of zo_score_static_capacity() bytes
 * (32 MiB) that every GPU the library runs on holds until the process ends.  The
 * call allocates nothing.  A batch whose scratch (zo_score_workspace_bytes) exceeds
 * the capacity is rejected with ZO_ERR_WORKSPACE before anything is launched: e.g.
 * 4096 tokens at a vocabulary of 151936, or 16384 tokens at 50272, still fit.  All
 * calls on one GPU share that GPU's array: calls that overlap in time on one GPU
 * (different streams, or different threads) race; calls on one stream do not.
 */
size_t zo_score_static_capacity(void);

int32_t zo_score_static(const zo_batch* batch, const void* H, int64_t ldh,
                        const void* W_head, int64_t ldw, int32_t vocab, int32_t d,
                        zo_dtype dtype, const int32_t* targets,
                        float* tok_nll, float* seq_nll, float* cand_sum, int32_t* cand_cnt,
                        void* stream);

/*
 * Antithetic two-point estimate (Sec. 2.1, Eq. 2):
 *   cand_loss[c] = cand_sum[c] / max(cand_cnt[c], 1)   (reduction 0, mean)
 *                = cand_sum[c]                          (reduction 1, sum)
 *   proj_grad[k] = (cand_loss[c+] - cand_loss[c-]) / (2 eps)
 * where c+ / c- are the lowest-numbered candidates of direction k with
 * positive / negative sign; a direction lacking either gets 0.
 * cand_loss fp32 [C], proj_grad fp32 [K]; needs no workspace.
 */
int32_t zo_estimate(const zo_batch* batch, const float* cand_sum, const int32_t* cand_cnt,
                    float eps, int32_t reduction, float* cand_loss, float* proj_grad,
                    void* stream);

/*
 * Reward-normalised one-sided estimate (Sec. 2.2, Sec. 5.3 and the taxonomy appendix: N candidate evaluations around
 * one centre, reward normalisation, reward-weighted update; the evolution-
 * strategies shape).  Direction k is represented by its lowest-numbered
 * candidate with positive sign, reward R_k = -cand_loss of that candidate;
 * over the N directions that have one,
 *   z_k = (R_k - mean R) / max(std R, 1e-8)    (population std, fixed-order sums)
 *   proj_grad[k] = -z_k / eps                  (0 for directions without one)
 * so that zo_bank_update's beta_k = -lr proj_grad[k] / N = lr z_k / (N eps).
 * The formula is this library's reading: the paper names the ingredients only.
 * Arguments as zo_estimate.
 */
int32_t zo_estimate_es(const zo_batch* batch, const float* cand_sum, const int32_t* cand_cnt,
                       float eps, int32_t reduction, float* cand_loss, float* proj_grad,
                       void* stream);

/*
 * Lazy bank update (Sec. 3.2, Eq. "layer-coupling": sum_t beta_t U_t V_k^T =
 * P_k V_k^T, so only P_k is maintained).  For every direction k, with
 * beta_k = -lr * proj_grad[k] * dir_weight[k] read on the device:
 *   append = 0:  P[:, col0[k] : col0[k]+r] += beta_k U_k
 *   append = 1:  P[:, block] = beta_k U_k;  Vb[:, block] = V_k
 * U_k is regenerated from dir_seed[k], V_k from dir_seed_v[k] (dir_seed[k]
 * when dir_seed_v is NULL); factor_dtype as in zo_probe_linear's in_dtype.
 * dir_weight NULL means 1/n_dirs.
 *   host_col0  HOST int32 [n_dirs]: first column of each direction's block;
 *              blocks must not overlap each other.
 * On append, bank->R_used (a host field) is raised to max(col0[k] + r).
 * Returns ZO_ERR_BANK_FULL when a block does not fit in R_cap.
 * W_0 is not an argument: the base is never touched.
 */
int32_t zo_bank_update(zo_bank* bank, int32_t m, int32_t n, int32_t r, int32_t n_dirs,
                       const uint64_t* dir_seed, const uint64_t* dir_seed_v, uint32_t tensor_id,
                       const float* proj_grad, float lr, const float* dir_weight,
                       const int32_t* host_col0, int32_t append, zo_dtype factor_dtype,
                       void* stream);

/*
 * The same lazy update for many layers in one call (Sec. 5.2, the state-transition traffic table, counts the update of the
 * whole model as one state transition of 26 MB): every layer gets beta_k U_k of its
 * own tensor id in the same column blocks host_col0[k] (and, with append, V_k).  One
 * layer's update moves 2 * m * r * 4 bytes, a few hundred KB at the paper's sizes, so
 * per-layer launches cost more than the traffic; here up to 48 layers and 32
 * directions share a launch.  Other arguments and errors as zo_bank_update; nothing
 * is launched unless every layer passes validation.
 */
typedef struct zo_layer_bank {
  zo_bank bank;
  int32_t m, n;          /* shape of the layer's weight */
  uint32_t tensor_id;
  int32_t reserved;
} zo_layer_bank;

int32_t zo_bank_update_multi(zo_layer_bank* layers, int32_t n_layers, int32_t r, int32_t n_dirs,
                             const uint64_t* dir_seed, const uint64_t* dir_seed_v,
                             const float* proj_grad, float lr, const float* dir_weight,
                             const int32_t* host_col0, int32_t append, zo_dtype factor_dtype,
                             void* stream);

/*
 * Device-resident schedule of the multi-step loop (Sec. 3.2: V_k reused over an
 * interval of nu steps, U_t fresh every step, one bank block per interval; with
 * B blocks the reuse covers nu * B steps before the bank must be folded or the
 * run stops).  The state lives in device memory so that a captured HIP graph of
 * one step can be replayed without any host update.
 *
 * zo_schedule_step reads t = sched->next_step and writes, for step t with
 * K = n_dirs directions:
 *     interval = t / nu,  block = interval % n_blocks,  append = (t % nu == 0)
 *     dir_seed[j]   = base_u + t * K + j          (mod 2^64)
 *     dir_seed_v[j] = base_v + interval * K + j   (mod 2^64)
 * then sched->step = t and sched->next_step = t + 1.  The numbering of seeds
 * and blocks is this library's own; the paper fixes none.  Wrapping onto a
 * block that still holds an earlier interval reopens it (that interval's
 * update is discarded): the caller stops or folds after nu * n_blocks steps.
 *   sched       DEVICE zo_sched; set next_step (usually 0) before the first call
 *   dir_seed, dir_seed_v  DEVICE uint64 [n_dirs], overwritten
 */
typedef struct zo_sched {
  int64_t next_step;
  int64_t step;
  int32_t interval;
  int32_t block;
  int32_t append;
  int32_t reserved;
} zo_sched;

int32_t zo_schedule_step(zo_sched* sched, int32_t nu, int32_t n_blocks, int32_t n_dirs,
                         uint64_t base_u, uint64_t base_v,
                         uint64_t* dir_seed, uint64_t* dir_seed_v, void* stream);

/*
 * zo_bank_update driven by the device-resident schedule: direction k updates
 * columns [(sched->block * n_dirs + k) * r, +r), opening the block
 * (P = beta U, Vb = V) when sched->append is set and accumulating otherwise.
 * The bank must span all blocks from the start: R_used >= n_blocks * n_dirs * r,
 * unopened blocks zero (ZO_ERR_BANK_FULL / ZO_ERR_SHAPE otherwise); R_used is
 * not changed.  sched is a DEVICE pointer; everything else as zo_bank_update.
 */
int32_t zo_bank_update_scheduled(zo_bank* bank, int32_t m, int32_t n, int32_t r, int32_t n_dirs,
                                 const uint64_t* dir_seed, const uint64_t* dir_seed_v,
                                 uint32_t tensor_id, const float* proj_grad, float lr,
                                 const float* dir_weight, const zo_sched* sched, int32_t n_blocks,
                                 zo_dtype factor_dtype, void* stream);

/*
 * Fold the bank into the base (Sec. 3.2: standalone runs may fold the external
 * state; Eq. "bank" read right to left):
 *   W <- W + P[:, :R_used] Vb[:, :R_used]^T      (fp32 arithmetic, one rounding to dtype)
 * and then zeroes those columns of P and Vb on the device: the bank represents
 * no update any more and its blocks can be reopened.  bank->R_used is left as
 * it is.  This is the ONLY entry point that writes base weights; W [m x n] ld ldw
 * of type dtype is read and written in place.
 */
int32_t zo_fold_bank(zo_bank* bank, void* W, int64_t ldw, int32_t m, int32_t n, zo_dtype dtype,
                     void* stream);

/*
 * ---- What joins the probe linears of a decoder block ------------------------
 * A candidate's scoring pass (Sec. 2.2: a query is a teacher-forced scoring
 * pass of the model under the candidate's weights) runs whole decoder blocks.
 * The probed tensors are the block's linear layers (Sec. 3.2); normalisation,
 * causal self-attention inside each packed sequence (Sec. 3.1) and the residual
 * sums carry no perturbed parameters, are the same for every candidate and so
 * take no candidate table.  The paper does not spell these operations out;
 * they follow the standard definitions of the model families it evaluates.
 */
typedef enum zo_norm { ZO_LAYER_NORM = 0, ZO_RMS_NORM = 1 } zo_norm;

/*
 * Residual sum and normalisation of packed rows:
 *   h = X + R                      (R NULL: h = X)
 *   ZO_LAYER_NORM  Y = (h - mean(h)) / sqrt(var(h) + norm_eps) * gamma + beta   (biased variance)
 *   ZO_RMS_NORM    Y = h / sqrt(mean(h^2) + norm_eps) * gamma                   (beta ignored)
 * X, R, Hsum, Y: [n_tokens x d] of type dtype with leading dimensions ldx,
 * ldr, ldh, ldy; gamma, beta: fp32 [d] (beta may be NULL).  Hsum (optional,
 * needs R) receives h rounded to dtype, and it is that rounded h which is
 * normalised; Hsum may alias X or R.  Y is optional (NULL: only the sum is
 * written); Hsum and Y may not both be NULL.  fp32 arithmetic, moments by the
 * two-pass formula.  No workspace.
 */
int32_t zo_add_norm(const void* X, int64_t ldx, const void* R, int64_t ldr,
                    const float* gamma, const float* beta, int32_t kind, float norm_eps,
                    int32_t n_tokens, int32_t d, zo_dtype dtype,
                    void* Hsum, int64_t ldh, void* Y, int64_t ldy, void* stream);

/*
 * Causal self-attention over the packed sequences of `batch` (only n_tokens,
 * n_seqs and cu_seqlens are read): for row t of sequence i and query head h,
 *   O[t, h] = sum_j softmax_j(scale * <Q[t, h], K[j, g]>) V[j, g],
 *   j over rows cu[i] .. t of the same sequence,  g = h / (n_heads / n_kv_heads).
 * Q, O: [n_tokens x n_heads*head_dim]; K, V: [n_tokens x n_kv_heads*head_dim];
 * each with its own leading dimension, so the three may be column ranges of
 * one fused projection output.  O must not overlap Q, K or V.
 * ZO_BF16: head_dim must be 128; products on bf16 MFMA with fp32 accumulation,
 * softmax in fp32, weights rounded to bf16 before the second product.
 * ZO_F32: head_dim <= 256, fp32 throughout.  No workspace.
 */
int32_t zo_attention(const zo_batch* batch, const void* Q, int64_t ldq, const void* K, int64_t ldk,
                     const void* V, int64_t ldv, int32_t n_heads, int32_t n_kv_heads,
                     int32_t head_dim, float scale, zo_dtype dtype, void* O, int64_t ldo,
                     void* stream);

/*
 * The extra joining operation of the Qwen3 family (standard definitions; the paper
 * evaluates Qwen3-8B but does not spell them out; the family's gated MLP is
 * activation 2 of zo_probe_linear).
 *
 * zo_qk_norm_rope, in place on the query and key rows (column ranges of the fused
 * projection output, as for zo_attention): per head
 *   x <- x / sqrt(mean(x^2) + norm_eps) * gamma          (gamma_q for queries, gamma_k for keys,
 *                                                         fp32 [head_dim]; both NULL: no norm)
 * and then the rotary embedding: with p the row's offset in its own sequence,
 *   (x[i], x[i + head_dim/2]) <- rotation of that pair by the angle p * rope_theta^(-2i/head_dim)
 * (rope_theta <= 0: no rotation).  head_dim even, <= 256; one rounding to dtype.
 */
int32_t zo_qk_norm_rope(const zo_batch* batch, void* Q, int64_t ldq, void* K, int64_t ldk,
                        int32_t n_heads, int32_t n_kv_heads, int32_t head_dim,
                        const float* gamma_q, const float* gamma_k, float norm_eps,
                        float rope_theta, zo_dtype dtype, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ZO_H_ */
