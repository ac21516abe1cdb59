/*
 * verillm.h - C ABI of the verification hot path on one AMD MI355X (gfx950).
 *
 * What the library does (VeriLLM, arXiv 2509.24257):
 *   - Section 4, Eq. (1), and Section 5.6 "Verification Scheme": a verifier that knows the whole
 *     sequence [prompt || y_1..T] re-runs it as ONE teacher-forced causal forward pass and thereby
 *     recovers the hidden state of every position at every segment boundary.
 *   - Section 5.7 "Comparison and On-Chain Commitment": the recomputed states S_hat are compared
 *     elementwise with the inferencer's committed states S (Delta = S_hat - S), reduced per token and
 *     thresholded; the tail additionally checks TokenMatch(argmax f_LM(S_hat), y).
 *   - Section 5.5 "Inference Scheme": the inferencer produced those commitments token by token
 *     (S_1 = Embed(x), S_{i+1} = F_i(S_i; W_i), y = Decode(S_{L+1})); vl_decode_commit plays that role.
 *
 * The paper leaves the block F_i abstract.  This library implements the Llama-style pre-norm decoder
 * block: RMSNorm, rotary embedding on half-split pairs (i, i + head_dim/2) with angle
 * pos * rope_base^(-2i/head_dim), grouped-query causal attention scaled by 1/sqrt(head_dim) (query head j
 * reads key/value head j / (n_q_heads / n_kv_heads)), SwiGLU feed-forward, no biases, a final RMSNorm and an
 * untied LM head.  "Hidden state after layer l" is the residual stream leaving block l (before any
 * following norm), for every l in [1, n_layers].
 *
 * Conventions
 *   - Every function returns VL_OK (0) or a negative vl_status; nothing throws across the boundary.
 *     vl_last_error() gives a message for the most recent failure on that context.
 *   - Pointers marked [device] are device memory owned by the caller (for example the data_ptr() of a
 *     PyTorch-ROCm tensor) on the context's device.  Pointers marked [host] are ordinary host memory.
 *     The library never keeps a caller pointer after the call returns.
 *   - All work is enqueued on the stream given to vl_create (NULL = the default stream).  Calls that
 *     return results to the host synchronise that stream once before returning.
 *   - All device memory (weights, workspace, KV cache, logits) is allocated inside vl_create; no other
 *     call allocates.  One context serves one call at a time.
 *   - Token rows are "packed": sequence b occupies rows [cu[b], cu[b] + lengths[b]) with
 *     cu[b] = lengths[0] + ... + lengths[b-1].  Attention is causal within a sequence and never crosses
 *     sequences.  N = sum(lengths).
 *   - Matrices are row-major.  Weight matrices are [out_features, in_features] (y = x W^T).
 *   - bf16 values are stored as their 16-bit patterns; every float -> bf16 conversion rounds to nearest,
 *     ties to even.
 *   - On error no output buffer may be trusted.
 */
#ifndef VERILLM_H
#define VERILLM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct vl_ctx vl_ctx;          /* opaque: owns device weights, workspace, KV cache */

typedef enum { VL_F32 = 0, VL_BF16 = 1 } vl_dtype;

typedef enum {
    VL_OK = 0,
    VL_E_ARG = -1,        /* null pointer, bad size, bad layer list, bad dtype ...              */
    VL_E_WEIGHTS = -2,    /* a compute call before every tensor has been loaded                */
    VL_E_CAPACITY = -3,   /* N, B or a sequence length beyond what vl_create was sized for      */
    VL_E_HIP = -4,        /* a HIP runtime call failed (message in vl_last_error)              */
    VL_E_NOMEM = -5       /* device or host allocation failed                                  */
} vl_status;

typedef enum {
    VL_T_EMBED = 0,       /* [vocab, d_model]                                   model dtype     */
    VL_T_ATTN_NORM = 1,   /* [d_model]  gain of the pre-attention RMSNorm       float32         */
    VL_T_WQ = 2,          /* [n_q_heads*head_dim, d_model]                      model dtype     */
    VL_T_WK = 3,          /* [n_kv_heads*head_dim, d_model]                                     */
    VL_T_WV = 4,          /* [n_kv_heads*head_dim, d_model]                                     */
    VL_T_WO = 5,          /* [d_model, n_q_heads*head_dim]                                      */
    VL_T_FFN_NORM = 6,    /* [d_model]  gain of the pre-FFN RMSNorm             float32         */
    VL_T_W_GATE = 7,      /* [d_ffn, d_model]                                                   */
    VL_T_W_UP = 8,        /* [d_ffn, d_model]                                                   */
    VL_T_W_DOWN = 9,      /* [d_model, d_ffn]                                                   */
    VL_T_FINAL_NORM = 10, /* [d_model]                                          float32         */
    VL_T_LM_HEAD = 11,    /* [vocab, d_model]                                   model dtype     */
    VL_T_COUNT = 12
} vl_tensor_kind;

typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    float   rms_eps, rope_base;
    int32_t dtype;          /* vl_dtype of the weights and of every GEMM operand; the residual stream,
                               all accumulators, norm statistics, softmax and logits are float32     */
    int32_t max_tokens;     /* largest N of any call                                                 */
    int32_t max_seqs;       /* largest B of any call                                                 */
    int32_t max_seq_len;    /* longest single sequence (sizes the rotary table)                      */
} vl_model_cfg;
/* VL_BF16 models need d_model, n_q_heads*head_dim and d_ffn to be multiples of 64 and head_dim == 128 or
   64 (matrix-core tile shapes).  VL_F32 models need d_model % 8 == 0, d_ffn % 16 == 0, head_dim % 4 == 0 and
   head_dim <= 256.  Every sequence of every call must satisfy lengths[b] <= max_seq_len. */

typedef struct {
    float rel_l2;        /* accept a committed layer at a token iff ||Delta||_2 / max(||S_hat||_2,1e-30) <= rel_l2 */
    float max_abs;       /* ... and max|Delta| <= max_abs  (+infinity disables this gate)                            */
    float logit_margin;  /* accept the committed token a* iff max_v z[v] - z[a*] <= logit_margin; 0 = the paper's
                            exact TokenMatch.  A positive margin keeps honest near-ties from flipping under
                            floating-point noise.                                                                    */
} vl_tol;

typedef struct {         /* per (committed layer, token); Delta = recomputed - committed */
    float rel_l2;        /* ||Delta||_2 / max(||S_hat||_2, 1e-30)       */
    float max_abs;       /* max |Delta|  (NaN if any element is NaN)    */
    float mean_abs;      /* mean |Delta|: the paper's example phi = MAE */
    float mean_signed;   /* mean Delta                                  */
} vl_tok_stats;

typedef struct {
    int64_t n_tokens, n_rejected, n_hidden_reject, n_token_reject;
    float   max_rel_l2, max_abs;   /* maxima over all committed layers and tokens, NaNs ignored           */
    float   mean_mae;              /* T_v of Section 5.7 with phi = MAE and Psi = mean over tokens/layers */
    float   ms_forward, ms_compare;/* device time of the call: everything, and the compare/argmax part    */
} vl_summary;

/* Section 7 "Bit-aware statistical comparison" and the offline test battery of Appendix A.1 (P_exp, Q_small,
   Z_large, MAE).  Both states are taken as canonical float32 (a bf16 record is upcast exactly) and split into the
   exponent field (bits 30..23) and the mantissa field (bits 22..0); Delta is the float32 difference
   recomputed - recorded; the sign bit enters no count.  Per token, over the d_model elements of a state:
     P_e = n_exp_mismatch / d
     P_m = n_mismatch_close / n_exp_mismatch      close: |Delta| <= e_w although the exponent fields differ
     P_w = n_match_small / (d - n_exp_mismatch)   small: mantissa fields at most e_m steps apart, one step being
                                                  2^step_log2 units of the float32 mantissa (0 for float32 records,
                                                  16 for bf16 records, whose mantissa has 7 bits)
     Q_small = n_small / d (|Delta| <= q_small),  Z_large = n_large / d (|Delta| > tau_large)
   The rule accepts a token iff P_e < pe_max, P_m > pm_min, P_w > pw_min, |mean Delta| <= eps_max,
   Q_small >= q_small_min and Z_large <= z_large_max; a ratio over an empty set passes; each ratio test is decided
   as count vs bound * size in float32.  The paper's calibrated off-chain values are pe_max 0.05, pm_min 0.75,
   pw_min 0.80, eps_max 0.01 with e_w = 1e-2, e_m = 7, q_small = 1e-5; q_small_min = 0 and z_large_max = 1 switch
   the two battery bounds off. */
typedef struct {
    float   e_w;
    int32_t e_m;                   /* >= 0 */
    int32_t step_log2;             /* 0 .. 23 */
    float   q_small, tau_large;
    float   pe_max, pm_min, pw_min, eps_max, q_small_min, z_large_max;
} vl_bit_rule;

typedef struct {
    int32_t  n_exact;              /* identical bit patterns */
    int32_t  n_exp_mismatch, n_mismatch_close, n_match_small, n_small, n_large;
    float    mean_signed;          /* mean Delta, as in vl_tok_stats */
    uint32_t ok;                   /* 1 iff the rule accepts the token at this layer */
} vl_bit_stats;

/* ---- life cycle ------------------------------------------------------------------------------- */

/* Validate `cfg` and report the device memory vl_create would allocate for it.  Host only; touches no GPU.
   Either output may be NULL.  VL_E_ARG on a null or invalid cfg. */
int vl_plan_memory(const vl_model_cfg* cfg /*[host]*/, uint64_t* weight_bytes, uint64_t* workspace_bytes);

/* Create a context on `device` and allocate everything.  `hip_stream` is a caller-owned hipStream_t (or
   NULL); it must outlive the context.  *out is set to NULL on failure (the message is then only available
   from vl_last_error(NULL)). */
int vl_create(const vl_model_cfg* cfg /*[host]*/, int device, void* hip_stream, vl_ctx** out);

/* Copy one tensor into the context.  `src` may be host or device memory holding exactly `nbytes` bytes in
   the layout and dtype listed at vl_tensor_kind; the caller may free it as soon as the call returns.
   `layer` is 0-based and ignored for EMBED / FINAL_NORM / LM_HEAD.  Tensors may arrive in any order, one
   at a time, so a large model never has to sit in host memory whole.  The library stores WQ/WK/WV as one
   fused matrix and W_GATE/W_UP interleaved in row blocks. */
int vl_load_weights(vl_ctx* ctx, int tensor_kind, int layer, const void* src, size_t nbytes);

void vl_destroy(vl_ctx* ctx);
const char* vl_last_error(const vl_ctx* ctx);   /* ctx may be NULL: last error of a failed vl_create */

/* ---- the hot path ----------------------------------------------------------------------------- */

/* Section 4 Eq. (1) + Section 5.7.  One causal prefill over the packed batch, compared on the fly:
 *   after block l in commit_layers: per-token statistics of Delta against committed_hidden[c] and
 *   ok_c[n] = (rel_l2 <= tol.rel_l2) && (max_abs <= tol.max_abs)  (a NaN/Inf commitment fails);
 *   if committed_argmax != NULL: logits, argmax (lowest index among equal maxima) and the token check;
 *   flags[n] = 1 (accept) iff every ok_c[n] and the token check hold, else 0.
 *
 * tokens            [device] int32 [N], ids in [0, vocab)
 * lengths           [host]   int32 [B], each >= 0; N = sum, N <= max_tokens, B <= max_seqs
 * commit_layers     [host]   int32 [C], 1-based, strictly ascending, within [1, n_layers]; C >= 0
 * committed_hidden  [device] [C][N][d_model] contiguous in `hidden_dtype` (VL_F32 or VL_BF16)
 * committed_argmax  [device] int32 [N] or NULL (no LM head is run); an entry of -1 skips that position,
 *                            any other id outside [0, vocab) fails it
 * tol               [host]
 * flags             [device] out uint8 [N]
 * stats             [device] out vl_tok_stats [C][N], or NULL
 * summary           [host]   out, or NULL
 * N == 0 is legal and does nothing. */
int vl_verify_prefill(vl_ctx* ctx,
                      const int32_t* tokens, const int32_t* lengths, int32_t B,
                      const int32_t* commit_layers, int32_t C,
                      const void* committed_hidden, int32_t hidden_dtype,
                      const int32_t* committed_argmax,
                      const vl_tol* tol,
                      uint8_t* flags, vl_tok_stats* stats, vl_summary* summary);

/* Section 5.6, segment-local form: the verifier of one layer segment recomputes only blocks start_layer+1 ..
 * end_layer.  For start_layer > 0 it starts from the states recorded at the upstream boundary (the inferencer's
 * commitment for layer start_layer, taken as given), so the verifiers of different segments need nothing from
 * each other; for start_layer == 0 it starts from the token embedding and `upstream_hidden` is ignored.
 * Everything else is vl_verify_prefill restricted to the segment:
 *
 * start_layer, end_layer   0 <= start_layer < end_layer <= n_layers
 * upstream_hidden  [device] [N][d_model] in `upstream_dtype` (VL_F32 or VL_BF16); upcast exactly to the fp32
 *                           residual stream.  Required when start_layer > 0.
 * tokens           [device] int32 [N]; required when start_layer == 0, otherwise unused and may be NULL
 * commit_layers    [host]   as above, every entry in (start_layer, end_layer]
 * committed_argmax [device] as above; allowed only when end_layer == n_layers (VL_E_ARG otherwise)
 * Only the tensors of blocks start_layer+1 .. end_layer (plus the embedding when start_layer == 0, plus the final
 * norm and LM head when committed_argmax != NULL) must have been loaded; VL_E_WEIGHTS otherwise.
 * flags / stats / summary as in vl_verify_prefill, stats indexed [c][n] over this call's commit_layers. */
int vl_verify_segment(vl_ctx* ctx, int32_t start_layer, int32_t end_layer,
                      const void* upstream_hidden, int32_t upstream_dtype,
                      const int32_t* tokens, const int32_t* lengths, int32_t B,
                      const int32_t* commit_layers, int32_t C,
                      const void* committed_hidden, int32_t hidden_dtype,
                      const int32_t* committed_argmax,
                      const vl_tol* tol,
                      uint8_t* flags, vl_tok_stats* stats, vl_summary* summary);

/* Section 5.6: the same prefill, but RETURNING the states instead of comparing them ("each verifier must
 * return its computed outputs through the same interface as during inference").
 * out_hidden [device] [C][N][d_model] in hidden_dtype, or NULL; out_argmax [device] int32 [N], or NULL
 * (NULL skips the LM head). */
int vl_prefill_commit(vl_ctx* ctx,
                      const int32_t* tokens, const int32_t* lengths, int32_t B,
                      const int32_t* commit_layers, int32_t C,
                      void* out_hidden, int32_t hidden_dtype, int32_t* out_argmax);

/* Section 5.5: the inferencer.  For each sequence the first prompt_lens[b] positions are processed as one
 * prefill that fills the KV cache; every later position is processed on its own, in generation order,
 * against the cache (prompt_lens NULL = all zero = every position token by token).  Teacher-forced on
 * `tokens`.  Writes the states that an honest inferencer would commit, in exactly the layout
 * vl_verify_prefill consumes.  Needs lengths[b] <= max_seq_len.
 * prompt_lens [host] int32 [B] or NULL, 0 <= prompt_lens[b] <= lengths[b]. */
int vl_decode_commit(vl_ctx* ctx,
                     const int32_t* tokens, const int32_t* lengths, const int32_t* prompt_lens, int32_t B,
                     const int32_t* commit_layers, int32_t C,
                     void* out_hidden, int32_t hidden_dtype, int32_t* out_argmax);

/* Switch the bit-aware rule on (rule != NULL; the struct is copied) or off (NULL, the default) for later
   vl_verify_prefill / vl_verify_segment calls on this context.  While on, every committed layer is additionally
   judged by the rule in the same pass over the data, a token's hidden check passes only if the tolerance test AND
   the rule pass at every committed layer, and the per-token counts are kept for vl_get_bit_stats.
   VL_E_ARG for e_m < 0, step_log2 outside [0, 23] or a NaN field. */
int vl_set_bit_rule(vl_ctx* ctx, const vl_bit_rule* rule);

/* Counts of commit-layer index c (0-based position in that call's commit_layers) for rows [tok_begin, tok_end) of
   the most recent verify call made while a rule was set: out [device] vl_bit_stats [tok_end - tok_begin].
   VL_E_ARG if that call had no rule, or c / the range is outside it. */
int vl_get_bit_stats(vl_ctx* ctx, int32_t c, int64_t tok_begin, int64_t tok_end, vl_bit_stats* out);

/* ---- inspection of the most recent vl_verify_prefill / vl_prefill_commit (parity checks) ------- */

/* Copy logits rows [tok_begin, tok_end) of the most recent call that ran the LM head: out [device] float32
   [(tok_end - tok_begin)][vocab].  VL_E_ARG if that call ran no LM head or the range is outside its N. */
int vl_get_logits(vl_ctx* ctx, int64_t tok_begin, int64_t tok_end, float* out);

/* Copy the recomputed argmax and the gap (max_v z[v] - z[committed]; 0 where skipped or where the call had
   no committed tokens) of rows [tok_begin, tok_end): out_argmax [device] int32, out_gap [device] float32,
   either may be NULL. */
int vl_get_argmax(vl_ctx* ctx, int64_t tok_begin, int64_t tok_end, int32_t* out_argmax, float* out_gap);

/* ---- per-stage device timing (measurement only; off by default) -------------------------------- */

typedef enum {
    VL_STAGE_EMBED = 0, VL_STAGE_NORM = 1, VL_STAGE_QKV_GEMM = 2, VL_STAGE_ROPE = 3, VL_STAGE_ATTENTION = 4,
    VL_STAGE_O_GEMM = 5, VL_STAGE_GATEUP_GEMM = 6, VL_STAGE_DOWN_GEMM = 7, VL_STAGE_COMPARE = 8,
    VL_STAGE_LM_GEMM = 9, VL_STAGE_ARGMAX = 10, VL_STAGE_FINALIZE = 11, VL_STAGE_COUNT = 12
} vl_stage;

/* mode 0: off.  mode 1: event pairs around the gate/up GEMM launches only (the kernel that carries half of
   the flops).  mode 2: around every stage of vl_verify_prefill / vl_prefill_commit.  Events are recorded on
   the context's stream and read when the call synchronises. */
int vl_profile_enable(vl_ctx* ctx, int mode);
/* Device milliseconds and launch counts per stage accumulated since the previous read; then reset.
   ms [host] double[VL_STAGE_COUNT], launches [host] int64[VL_STAGE_COUNT]; either may be NULL. */
int vl_profile_read(vl_ctx* ctx, double* ms, int64_t* launches);

/* ---- single operations, exposed so that each kernel can be checked on its own ------------------ */

/* C[M,N] = A[M,K] * W[N,K]^T on the matrix cores: A, W bf16 [device], fp32 accumulate, `out` bf16 when
   out_dtype == VL_BF16 else float32.  K must be a multiple of 64; M, N >= 1.  M <= 64 rows take the weight-streaming
   kernel of the token-by-token path, larger M the 256 x 256 tile kernel of the prefill. */
int vl_op_gemm_bf16(vl_ctx* ctx, const void* A, const void* W, void* out, int32_t out_dtype,
                    int32_t M, int32_t N, int32_t K);

/* Causal grouped-query attention over packed sequences on the matrix cores.
   qkv [device] bf16 [N][(n_q_heads + 2 n_kv_heads) * head_dim] holding, per token, the query heads, then
   the key heads, then the value heads (rotary embedding already applied to queries and keys).
   out [device] bf16 [N][n_q_heads * head_dim].  lengths [host] int32 [B]. */
int vl_op_attention_bf16(vl_ctx* ctx, const void* qkv, const int32_t* lengths, int32_t B, void* out);

/* The attention of one token-by-token step (Section 5.5) on its own: query row r attends to the n_keys[r] cached
   positions first_row[r] .. first_row[r] + n_keys[r] - 1 (its own key is the last of them).  bf16 contexts with
   head_dim 64 or 128 and n_q_heads / n_kv_heads in {1, 2, 4, 8}.
   q [device] bf16 [rows][n_q_heads*head_dim] (rotary embedding already applied); k_cache, v_cache [device] bf16
   [cache_rows][n_kv_heads*head_dim]; first_row, n_keys [host] int32 [rows], n_keys >= 1; out [device] bf16
   [rows][n_q_heads*head_dim].  VL_E_ARG if a key range leaves the cache. */
int vl_op_attention_decode_bf16(vl_ctx* ctx, const void* q, const void* k_cache, const void* v_cache, int64_t cache_rows,
                                const int32_t* first_row, const int32_t* n_keys, int32_t rows, void* out);

/* Compare stage alone (Section 5.7): h_hat [device] float32 [N][d_model] against committed [device]
   [N][d_model] in hidden_dtype; stats [device] out [N]; ok [device] out uint8 [N]. */
int vl_op_compare(vl_ctx* ctx, const float* h_hat, const void* committed, int32_t hidden_dtype, int64_t N,
                  const vl_tol* tol, vl_tok_stats* stats, uint8_t* ok);

/* Row argmax + token check alone: logits [device] float32 [N][vocab]; committed_argmax [device] int32 [N]
   or NULL; outputs [device], any may be NULL. */
int vl_op_argmax(vl_ctx* ctx, const float* logits, int64_t N, const int32_t* committed_argmax, float margin,
                 int32_t* out_argmax, float* out_gap, uint8_t* out_ok);

/* ---- Merkle commitment of hidden states (Section 5.6 "Commitment Submission", Section 5.7 MerkleVerify) ---------
 * A state row (d_model scalars) is serialised as canonical float32 (a bf16 row is upcast exactly), little endian.
 * Leaf j = SHA-256 of the 4 bytes of element j; inner node = SHA-256(left || right); a node without a right
 * neighbour at its level moves up unchanged; the root is the last node left.  Digests are 32 bytes, in the order
 * SHA-256 defines them. */
#define VL_MERKLE_DIGEST_BYTES 32
#define VL_MERKLE_MAX_OPENINGS 64

/* roots [device] out uint8 [rows][32]: the root of every row of states [device] [rows][d_model] in `dtype`.
   Any number of rows (for the states of C committed layers pass rows = C * N).  d_model <= 16384. */
int vl_op_merkle_roots(vl_ctx* ctx, const void* states, int32_t dtype, int64_t rows, uint8_t* roots);

/* Inclusion proofs for K <= VL_MERKLE_MAX_OPENINGS disclosed scalars: opening q is element sel_index[q] of row
   sel_row[q] (both [host]) of states [device] [rows][d_model].
   values   [device] out float32 [K], the disclosed scalars, or NULL
   paths    [device] out uint8 [K][depth][32] with depth = ceil(log2 d_model): the sibling digests from the leaf level
            upwards; a level where the node has no sibling contributes nothing, and entries past the proof are zero
   path_len [host]   out int32 [K], the number of digests of each proof, or NULL
   The receiver recomputes the root from (value, index, d_model, path). */
int vl_op_merkle_open(vl_ctx* ctx, const void* states, int32_t dtype, int64_t rows, const int64_t* sel_row,
                      const int32_t* sel_index, int32_t K, float* values, uint8_t* paths, int32_t* path_len);

/* vl_op_compare plus the bit-aware rule on the same rows: h_hat [device] float32 [N][d_model], committed [device]
   [N][d_model] in hidden_dtype; stats [device] out vl_tok_stats [N] or NULL, bits [device] out vl_bit_stats [N] or
   NULL, ok [device] out uint8 [N] (tolerance test AND rule) or NULL. */
int vl_op_compare_bits(vl_ctx* ctx, const float* h_hat, const void* committed, int32_t hidden_dtype, int64_t N,
                       const vl_tol* tol, const vl_bit_rule* rule, vl_tok_stats* stats, vl_bit_stats* bits, uint8_t* ok);

#ifdef __cplusplus
}
#endif
#endif /* VERILLM_H */
