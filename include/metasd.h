/*
 * metasd.h - C ABI of the MI355X (gfx950) MetaSD hot-path library.
 *
 * One round of MetaSD (Alg. 1 of the paper) is
 *     k = metasd_bandit_select()            Alg. 2, selection line / initial sweep
 *     metasd_draft(k, gamma)                Alg. 3, drafting loop: gamma tokens from drafter k
 *     metasd_verify(gamma)                  Alg. 3, "in parallel compute E+1 sets of logits"
 *     metasd_accept(gamma, ...)             Alg. 3, accept test / residual resample / bonus token
 *     metasd_bandit_update(k, n_acc, ...)   Alg. 2, mean update with the BE (or BD, Def. 2) reward
 *
 * Conventions
 *   - Every function returns 0 on success or a negative METASD_E_* code; nothing is thrown or
 *     aborted across this boundary.  metasd_last_error() gives a message for the last failure.
 *   - "device" pointers are HIP device memory owned by the CALLER (weights, KV caches,
 *     workspace); the library never allocates or frees device memory.  "host" pointers are
 *     ordinary host memory.  The library owns only its host-side context and one small
 *     pinned host buffer for results.
 *   - All device work is enqueued on the HIP stream given to metasd_create (NULL = default
 *     stream); draft and verify are asynchronous, accept synchronises the stream.
 *   - A context holds config.batch independent sequences (1..METASD_MAX_BATCH), each with its own
 *     token history, KV caches and bandit; they advance in lock-step, one round per
 *     draft / verify / accept call: every sequence drafts with its own arm (sequences that share
 *     an arm share that drafter's forward pass; drafters of one shape - bf16, head_dim >= 64 - share one
 *     forward pass per step across arms, with the same results), one verification block holds all
 *     batch x (gamma + 1) rows, one accept launch tests them all.  Sequence b uses Philox sequence
 *     id b.  batch == 1 runs the single-sequence kernels; metasd_accept_logits and
 *     metasd_sample_logits take any number of rows.
 *
 * Model weights.  A model is described by metasd_model_desc and a table of device pointers in
 * this order: embed [V][d]; per layer: attn_norm [d], wq [H*hd][d], wk [KH*hd][d],
 * wv [KH*hd][d], wo [d][H*hd], ffn_norm [d], w_gate [f][d] (NULL when act == GELU),
 * w_up [f][d], w_down [d][f]; then final_norm [d], lm_head [V][d].  hd = d / H.
 *   dtype METASD_F32: every tensor is float, matrices row-major [out][in].
 *   dtype METASD_BF16: every tensor is bf16; embed and the norm gains are plain row-major, every
 *     matrix (wq .. w_down, lm_head) must be in the library's streaming-tile order produced by
 *     metasd_pack_weight (same byte size as the row-major matrix; wq and wk with rope_head_dim = hd).
 *
 * KV cache of a model (device, caller-owned): element type = model dtype, one cache per sequence,
 *     [sequence][layer][2 (K, V)][kv_head][max_ctx][hd],  bytes = batch * metasd_kv_bytes().
 *
 * Drafter-switch KV strategies (the paper's appendix on switching costs and on efficient KV-cache strategies).
 *   default: every drafter has a cache of its own; when it is selected it first consumes the committed tokens it
 *     has not processed (the recomputation on a switch that the paper describes as its default).
 *   shared:  drafter_kv[k] == target_kv declares drafter k an early-exit drafter - its layers are the target's first
 *     n_layers layers (the same weight pointers; checked) followed by norm and head tensors of its own.  The K/V of
 *     those layers at committed positions are the numbers the target's cache already holds, so the drafter reads them
 *     there, never consumes a backlog, and writes the K/V of the positions it drafts into the shared cache, where the
 *     verification pass then writes the same values again.  Nothing is recomputed on a switch.
 */
#ifndef METASD_H
#define METASD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define METASD_OK 0
#define METASD_E_INVALID (-1)   /* bad argument: NULL, k out of range, gamma out of range, unsupported shape */
#define METASD_E_OVERFLOW (-2)  /* the KV cache / token history would exceed max_ctx */
#define METASD_E_ORDER (-3)     /* call-order violation (e.g. verify before draft) */
#define METASD_E_HIP (-4)       /* a HIP call failed; message retained */
#define METASD_E_WORKSPACE (-5) /* workspace too small; required size in the message */

#define METASD_GELU 0
#define METASD_SWIGLU 1
#define METASD_F32 0
#define METASD_BF16 1
#define METASD_REWARD_BE 0 /* block efficiency  N_acc / N_max */
#define METASD_REWARD_BD 1 /* block divergence, Def. 2 */

/* Drafter-selection policy.  UCB is Alg. 2 (MetaSD-UCB); the others are the paper's appendix
 * "Extensions" (switching costs, non-stationary rewards) and its EXP3 / random baselines. */
#define METASD_POLICY_UCB 0    /* Alg. 2 */
#define METASD_POLICY_DUCB 1   /* discounted UCB: policy_param = discount in (0, 1] */
#define METASD_POLICY_SWUCB 2  /* sliding-window UCB: policy_window = window length in rounds (>= 1) */
#define METASD_POLICY_EXP3 3   /* EXP3: policy_param = mixing gamma in (0, 1]; draws from Philox stream 3 */
#define METASD_POLICY_SH 4     /* sequential halving over policy_window rounds, then the survivor for good
                                  (pure exploration-then-commit with the exploration budget in rounds) */
#define METASD_POLICY_RANDOM 5 /* uniform random arm; Philox stream 3 */
#define METASD_MAX_GAMMA 15 /* a verification block is gamma+1 <= 16 rows */
#define METASD_MAX_K 64
#define METASD_MAX_BATCH 32 /* sequences per context; a verification block has batch * (gamma+1) <= 512 rows */

typedef struct metasd_ctx metasd_ctx; /* opaque; freed by metasd_destroy */

typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, d_ffn, vocab;
    int32_t act;   /* METASD_GELU | METASD_SWIGLU */
    int32_t dtype; /* METASD_F32 | METASD_BF16 */
    float rms_eps, rope_theta;
} metasd_model_desc;

typedef struct {
    int32_t K;          /* number of drafters, 1..METASD_MAX_K */
    int32_t gamma_max;  /* largest draft length N_max that will be used, 1..METASD_MAX_GAMMA */
    int32_t batch;      /* independent sequences in this context, 1..METASD_MAX_BATCH */
    int32_t max_ctx;    /* capacity of the token history and of every KV cache, in positions */
    float temperature;  /* 0 => greedy; otherwise p = softmax(logits / T) for target and drafter */
    int32_t reward;     /* METASD_REWARD_BE | METASD_REWARD_BD (used by metasd_bandit_update) */
    double ucb_beta;    /* exploration strength beta of Alg. 2 */
    uint64_t seed;      /* Philox key of all uniforms */
    int32_t policy;        /* METASD_POLICY_*; 0 (UCB) for a zero-initialised tail */
    int32_t policy_window; /* SWUCB: window; SH: exploration budget in rounds; else ignored */
    double policy_param;   /* DUCB: discount; EXP3: gamma; else ignored */
    /* Streaming drafter caches (the KV strategy of the paper's appendix "MetaEagle-UCB with efficient KV cache strategies",
     * which names the StreamingLLM technique and gives no sizes).  stream_window == 0: off - a drafter that is switched in
     * recomputes the K/V of every committed token it has not seen.  stream_window = W > 0 (batch == 1 only): every drafter
     * with a cache of its own attends, at position p, to the first stream_sink positions and to the last W positions up to
     * p, at their original positions; when it is switched in it consumes the sinks it has not seen and the last W
     * committed tokens only - a longer backlog is skipped and never attended to.  The drafter's distribution changes, the
     * output law does not (Alg. 3 is exact for any drafter). */
    int32_t stream_sink;
    int32_t stream_window;
    /* 1: the context keeps the target's hidden states ("features": the residual stream after the last layer) of every
     * processed position, for drafters that run on them (metasd_set_drafter_head).  batch == 1 only; costs max_ctx *
     * d_model * 4 bytes of workspace. */
    int32_t feature_heads;
} metasd_config;

/* ---- sizes -------------------------------------------------------------------------------- */

/* Bytes of one model's KV cache for ONE sequence of max_ctx positions (a context needs batch times this,
 * sequence b's cache starting b * bytes into the buffer). */
int32_t metasd_kv_bytes(const metasd_model_desc* m, int32_t max_ctx, size_t* bytes_out);

/* Bytes of device workspace metasd_create needs for this configuration. */
int32_t metasd_workspace_bytes(const metasd_config* cfg, const metasd_model_desc* target,
                               const metasd_model_desc* drafters /*[K]*/, size_t* bytes_out);

/* Re-order a row-major bf16 matrix W[n_out][n_in] (device) into streaming-tile order (device,
 * n_out*n_in*2 bytes, must not alias src): 1 KiB tiles of 16 output rows x 32 inputs, tile
 * (t, c) at ((t * n_in/32) + c) KiB, lane l of a wavefront owning bytes [16 l, 16 l + 16) =
 * W[16 t + l%16][32 c + 8 (l/16) .. +8].  Requires n_out % 16 == 0 and n_in % 32 == 0.
 * rope_head_dim: 0 for every matrix except the q and k projections, which pass the head
 * dimension hd: inside each head the rows are then re-ordered so that the two members (i, i + hd/2)
 * of a rotary pair sit next to each other (packed row 16 j + c of a head <- source row 8 j + c/2,
 * plus hd/2 when c is odd); the library undoes this when it writes q and the K cache.
 * Asynchronous on `hip_stream`. */
int32_t metasd_pack_weight(void* dst, const void* src, int32_t n_out, int32_t n_in, int32_t rope_head_dim, void* hip_stream);

/* ---- context ------------------------------------------------------------------------------ */

/* Create a context.  Descriptors and pointer tables are copied; the device memory they point
 * to stays owned by the caller and must outlive the context.  target_kv / drafter_kv[k] are
 * KV caches of batch * metasd_kv_bytes() each; workspace is >= metasd_workspace_bytes() and 256-byte
 * aligned.  Errors: INVALID (NULL, unsupported shape: see metasd_last_error), WORKSPACE, HIP. */
int32_t metasd_create(metasd_ctx** out, const metasd_config* cfg, const metasd_model_desc* target,
                      const metasd_model_desc* drafters /*[K]*/, const void* const* target_weights,
                      const void* const* const* drafter_weights /*[K] tables*/, void* target_kv,
                      void* const* drafter_kv /*[K]*/, void* workspace, size_t workspace_bytes, void* hip_stream);
int32_t metasd_destroy(metasd_ctx*);

/* Start a new query for sequence seq (Alg. 1 input "initial prompt x^{1:l}"): upload n >= 1 prompt
 * tokens (host) and reset that sequence's bandit (the bandit is re-initialised for every query) and its
 * round counter (the round word of its Philox counters: every sequence counts the rounds of its own
 * query, so re-setting one sequence of a batch leaves the uniforms of the others untouched).  A round
 * can be drafted once every sequence has a context; between metasd_draft and metasd_accept the call is
 * refused (ORDER).
 * kv_prefilled == 0: the target prefills positions [0, n-1) now (asynchronously); drafters start
 *   empty and catch up the first time they are selected.
 * kv_prefilled != 0: the caller has already written the KV entries of positions [0, n-1) of
 *   the target and of every drafter (synthetic or externally computed context).
 * Errors: INVALID, OVERFLOW (n + gamma_max + 1 > max_ctx), ORDER, HIP. */
int32_t metasd_set_context(metasd_ctx*, int32_t seq, const int32_t* tokens, int32_t n, int32_t kv_prefilled);

/* Replace entry `index` of the weight table of model `model` (-1 = target, k = drafter k) with
 * another device pointer of the same shape and layout (e.g. a drafter's LM head). */
int32_t metasd_swap_weight(metasd_ctx*, int32_t model, int32_t index, const void* dev_ptr);

/* ---- bandit (host, fp64; Alg. 2) ------------------------------------------------------------ */

/* Arm for the next round.  UCB (Alg. 2): arms 0..K-1 once each in index order, afterwards
 * argmax_i mu_i + beta * sqrt(2 ln t / n_i), t = completed rounds, lowest index on ties.
 * DUCB / SWUCB: the same index on discounted / windowed estimates (an arm without a pull in the
 * window is tried first).  EXP3: draw from (1 - g) w_i / sum w + g / K.  SH: the surviving arms in
 * turn, each floor(T / (|S| ceil(log2 K))) (at least 1) times per phase, the better half kept.
 * Call once per round: EXP3 keeps the probabilities of the latest call for the update. */
int32_t metasd_bandit_select(metasd_ctx*, int32_t seq, int32_t* k_out);
/* Feed back the round's reward to arm k: BE reward n_acc / gamma, or, when the context was
 * created with METASD_REWARD_BD, bd_reward (the value metasd_accept reported).  mu_k becomes
 * (mu_k n_k + r)/(n_k + 1), n_k and t advance (UCB; the other policies update as their
 * algorithms state).  Errors: INVALID. */
int32_t metasd_bandit_update(metasd_ctx*, int32_t seq, int32_t k, int32_t n_acc, int32_t gamma, double bd_reward);
/* Copy out mu[K], n[K], t (any pointer may be NULL): the estimates and counts the policy's index
 * uses (UCB, DUCB, SWUCB) or the plain per-arm mean reward and pull count (EXP3, SH, RANDOM). */
int32_t metasd_bandit_state(const metasd_ctx*, int32_t seq, double* mu, int32_t* n, int32_t* t);

/* ---- one speculative-sampling round (Alg. 3) -------------------------------------------------- */

/* Draft gamma tokens for every sequence b with drafter k[b]: the drafter first consumes the committed tokens it has
 * not processed yet (ending with the last committed token), then runs gamma-1 single-token steps.
 * Token j is argmax (T = 0) or the inverse-CDF draw of softmax(logits/T) with the Philox uniform
 * at (seq, round, j, stream 2).  Draft tokens and drafter logits stay on the device.
 * Errors: INVALID (k, gamma), OVERFLOW, ORDER (no context set / round already drafted), HIP. */
int32_t metasd_draft(metasd_ctx*, const int32_t* k /*[batch] host*/, int32_t gamma);

/* Target forward over the gamma+1 rows [last committed token, d_1 .. d_gamma] at positions
 * l-1 .. l-1+gamma against the KV cache (causal inside the block); appends their K/V and leaves
 * fp32 logits [batch][gamma+1][V] on the device.  Errors: INVALID, ORDER (draft not done), HIP. */
int32_t metasd_verify(metasd_ctx*, int32_t gamma);

/* Accept test u_j < min(1, p_j(d_j)/q_j(d_j)) for j < gamma with the uniform at (seq, round, j,
 * stream 0); N_acc = index of the first failure (gamma if none); the emitted token is drawn by
 * inverse CDF with the uniform at (seq, round, 0, stream 1) from norm(max(0, p_n - q_n)) if
 * n < gamma, else from p_gamma (greedy: accept iff d_j == argmax, emit argmax).  Synchronises,
 * then commits: history, KV lengths, round counter.  Outputs are host arrays of `batch` entries
 * (mask_out: bit j = raw test j; bd_out: mean over j of sum_v min(p_j, q_j)); any may be NULL.
 * If the workgroups of a position fail to meet within their bounded wait the step is taken again with
 * one workgroup per position before anything is committed (counted by metasd_accept_fallbacks).
 * Errors: INVALID, ORDER (verify not done), HIP (a split-K reduction of the forward passes timed out:
 * the round's state is lost, call metasd_set_context for every sequence to start over). */
int32_t metasd_accept(metasd_ctx*, int32_t gamma, int32_t* n_acc_out, int32_t* token_out, uint32_t* mask_out,
                      double* bd_out);

/* ---- drafter heads on the target's hidden states (the white-box drafters of the paper's Sec. 4, "Eagle") ------------
 * The paper gives no formulas for them; the reading, after the published design it cites: the feature f_p of position p is
 * the target's residual stream after its last layer at p.  A head processes position p from the token there and the
 * feature of the position before:  h = W_fc . [embedding(x_p) ; f_{p-1}]  (f_{-1} = 0, no bias), then its own decoder
 * layer(s) with a KV cache of its own; the result is its estimate of f_p, and final norm + LM head (its table entries:
 * normally the target's tensors) turn it into the distribution of x_{p+1}.  While drafting, the estimate is the feature
 * input of the next step; what was computed from estimates is dropped after the round, and the next time the head is
 * selected it first consumes the committed tokens since then with the target's own features.
 *
 * metasd_set_drafter_head marks drafter k (same width and dtype as the target; weight table as for any model, embedding
 * entry = the table the head embeds tokens with) as such a head.  w_fc: device pointer, [d_model][2 d_model], fp32
 * row-major or bf16 in streaming-tile order (metasd_pack_weight(n_out = d, n_in = 2 d, rope 0)), caller-owned.  Call it
 * after metasd_create and before the first metasd_set_context; the context must have feature_heads = 1.  With
 * kv_prefilled contexts the caller also fills the feature table (METASD_PEEK_FEAT) for the prefilled positions.
 * In tree rounds (metasd_draft_tree) a node takes the head's estimate at its parent; the target's features of the root and
 * of the accepted nodes are kept.  Errors: INVALID, ORDER. */
int32_t metasd_set_drafter_head(metasd_ctx*, int32_t k, const void* w_fc);

/* ---- multi-candidate rounds: a tree of draft tokens verified in one pass with tree attention -----------------------
 * (the white-box setting of the paper's Sec. 4, "Number of drafts": multi-draft methods verify a token tree).  The paper
 * states no rule for trees; what it fixes is losslessness (the paragraph after Alg. 3), and the rules here are the ones
 * that keep it:
 *   T = 0: the output must be the target's own greedy continuation, so the children of a node are the drafter's most
 *          likely next tokens and the accepted nodes are the longest path from the root on which every token is the
 *          target's most likely next token;
 *   T > 0: the children of a node, in ascending rank, are successive draws WITHOUT replacement from
 *          q = softmax(Q_node / T); verification is recursive rejection sampling (Jeon et al., "Recursive speculative
 *          decoding", 2024): at the current node with p = softmax(P_node / T), for each child in rank order with token
 *          x: accept with probability min(1, p(x) / q(x)) and move there; on a rejection p <- norm(max(0, p - q)) and
 *          q <- q with q(x) = 0, renormalised; when no child is accepted (or at a leaf) the emitted token is a draw
 *          from the current p.  With one child per node this is Alg. 3.  Philox counters: child node v uses position
 *          v - 1 (stream 2 for its draw, stream 0 for its test), the emitted token position 0 of stream 1 - a
 *          chain-shaped tree consumes exactly the counters of metasd_draft / metasd_accept.
 *
 * The tree's SHAPE is the caller's: node 0 is the root (the last committed token); node i > 0 is a child of node
 * parent[i] < i with rank rank[i]: for T = 0 the rank[i]-th most likely next token by the drafter's logits (0 = most
 * likely, ties to the lower token), for T > 0 the children of a node are drawn in ascending rank (only the order of the
 * ranks matters).  Nodes come in breadth-first order (depth never decreases), 2 <= n <= min(16, gamma_max + 1), and
 * the nodes above the deepest level number at most gamma_max.  A chain (parent[i] = i - 1, rank 0) is ordinary
 * speculation. */
#define METASD_MAX_TREE 16
typedef struct {
    int32_t n;
    int32_t parent[METASD_MAX_TREE]; /* parent[0] ignored */
    int32_t rank[METASD_MAX_TREE];   /* 0 .. 7; rank[0] ignored */
} metasd_tree;

/* Drafter k fills the tree level by level: one forward pass per level over that level's nodes (each node attends to
 * the committed tokens and to its own ancestors, and is rotated for position l - 1 + depth), then the children of
 * every node of the level get their tokens.  The first pass consumes the drafter's backlog of committed tokens as in
 * metasd_draft.  Contexts with batch == 1 only.
 * Errors: INVALID (shape, k, batch > 1), OVERFLOW, ORDER, HIP. */
int32_t metasd_draft_tree(metasd_ctx*, int32_t k, const metasd_tree* tree);
/* One target pass over all n nodes with the same tree attention; node i's K/V go to cache slot l - 1 + i for now;
 * fp32 logits [n][V] on the device (METASD_PEEK_P).  Errors: ORDER, HIP. */
int32_t metasd_verify_tree(metasd_ctx*);
/* Acceptance.  T = 0: from the root, step to the child that carries the target's most likely token, as long as there is
 * one; N_acc = steps taken, emitted token = the target's most likely token at the last node reached.  T > 0: the walk
 * described above (what happens at a node does not depend on how the walk got there: one workgroup per node decides
 * it, a last small kernel follows the decisions from the root).  The K/V of the
 * accepted nodes are moved from their tree slots to their positions (target and drafter caches), history, KV lengths
 * and round counter are committed.  path_out (host, may be NULL): the accepted nodes, N_acc entries.  The BE reward of
 * the round is N_acc / (depth of the tree): pass that depth as `gamma` to metasd_bandit_update.
 * Synchronises.  Errors: ORDER, HIP. */
int32_t metasd_accept_tree(metasd_ctx*, int32_t* n_acc_out, int32_t* token_out, int32_t* path_out);

/* ---- stand-alone kernels on caller-supplied logits (device) ------------------------------------ */

/* Accept step on rows of logits: P [rows][gamma+1][V], Q [rows][gamma][V] fp32, d [rows][gamma]
 * int32, all device.  Row b uses the uniforms of sequence id seq0 + b at `round`.  Outputs
 * (device, any of mask/bd may be NULL): n_acc [rows], token [rows], mask [rows] (bit j), bd
 * [rows][gamma] doubles (sum_v min(p_j, q_j)).  scratch: device, METASD_ACCEPT_SCRATCH_BYTES(rows, gamma)
 * bytes, zero-filled before its first use; later calls may reuse it as it is (each launch tags what
 * it writes there with a process-wide launch number), but two launches that overlap in time must not
 * share it.  A token of -2 reports that the four workgroups of a position did not meet within the
 * kernel's bounded wait (nothing hangs; the result of that row is invalid).
 * Requires V % 4 == 0 and V <= 32768.  Asynchronous on hip_stream. */
#define METASD_ACCEPT_SCRATCH_BYTES(rows, gamma) ((size_t)(rows) * ((size_t)(gamma) + 1) * 336)
int32_t metasd_accept_logits(const float* P, const float* Q, const int32_t* d, int32_t rows, int32_t gamma,
                             int32_t V, float temperature, uint64_t seed, uint32_t round, uint32_t seq0,
                             int32_t* n_acc, int32_t* token, uint32_t* mask, double* bd, void* scratch,
                             void* hip_stream);

/* The same step for callers that cannot allocate device memory or pass a workspace of their own (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): no scratch argument - the candidates
 * and exchange words live in an array built into the library, METASD_ACCEPT_NOALLOC_MAX_ITEMS * 336 bytes
 * (1.3 MiB) that every GPU the library runs on holds until the process ends.  Calls with
 * rows * (gamma + 1) > METASD_ACCEPT_NOALLOC_MAX_ITEMS are refused (INVALID; use metasd_accept_logits).  The
 * call allocates nothing and synchronises nothing: it enqueues one small kernel that clears the part of the array it
 * uses (the array keeps the last call's contents) and the accept kernel, on hip_stream of the current device.
 * All calls on one GPU share the array: two calls whose kernels overlap in time race.  Inputs, outputs, results and
 * errors otherwise as metasd_accept_logits. */
#define METASD_ACCEPT_NOALLOC_MAX_ITEMS 4096
int32_t metasd_accept_logits_noalloc(const float* P, const float* Q, const int32_t* d, int32_t rows, int32_t gamma,
                                     int32_t V, float temperature, uint64_t seed, uint32_t round, uint32_t seq0,
                                     int32_t* n_acc, int32_t* token, uint32_t* mask, double* bd, void* hip_stream);

/* Token draw per row of logits [rows][V] (device): argmax for T = 0, else inverse CDF of
 * softmax(logits/T) with the uniform at (seq0 + row, round, pos, stream 2).  tok [rows] device. */
int32_t metasd_sample_logits(const float* logits, int32_t rows, int32_t V, float temperature, uint64_t seed,
                             uint32_t round, uint32_t pos, uint32_t seq0, int32_t* tok, void* hip_stream);

/* Raw Philox4x32-10 output words for counters (c0_start + i, c1, c2, c3), i < n, key = seed:
 * out [n][4] uint32 device.  Used to check the generator against another implementation. */
int32_t metasd_philox_words(uint64_t seed, uint32_t c0_start, int32_t n, uint32_t c1, uint32_t c2, uint32_t c3,
                            uint32_t* out, void* hip_stream);

/* ---- measurement aids: not part of the method's boundary (no step of Alg. 1-3 needs them); benchmarks use them to
 * state achieved bandwidth per kernel next to what the machine reaches on a plain read ------------------------- */

/* One plain streaming read of src[0, bytes) (device, 16-byte aligned; bytes is rounded down to a
 * multiple of 1024, at least 1024) on the given stream, so that a benchmark can state the read rate this machine reaches next to the
 * nominal HBM peak.  sink: METASD_STREAM_READ_SINK_WORDS uint32 words of device memory that receive a digest of
 * what was read (the caller's; contents are of no use).  Asynchronous; the caller times it with events. */
#define METASD_STREAM_READ_SINK_WORDS 8192
int32_t metasd_stream_read(const void* src, size_t bytes, uint32_t* sink, void* hip_stream);

/* per-kernel timing */

#define METASD_PROF_GEMM 0   /* bf16 weight-streaming GEMM launches */
#define METASD_PROF_ATTN 1   /* KV-cache attention (partial) launches */
#define METASD_PROF_ACCEPT 2 /* the per-position accept kernel of metasd_accept */
/* max_records > 0: from now on every launch of the bandwidth-bound kernels carries a pair of HIP
 * events attached to the dispatch itself (begin and end of that kernel on the context's stream).  At most
 * max_records launches are recorded; the event pool is created here, not in the hot path, and
 * the record count is reset.  0: stop recording. */
int32_t metasd_profile(metasd_ctx*, int32_t max_records);
/* Synchronise and sum over the recorded launches of one kind: elapsed milliseconds, number of
 * launches, algorithmic bytes (weights / KV / logits each counted once per launch, plus the
 * small activation traffic).  Any output may be NULL. */
int32_t metasd_profile_read(metasd_ctx*, int32_t kind, double* ms_total, int64_t* launches, double* bytes_total);

/* The recorded weight-streaming GEMM launches grouped by shape (N output features, K inputs, m rows): summed
 * milliseconds, launches and algorithmic bytes per shape, in order of first appearance; target_only != 0 leaves out
 * the drafters' launches.  At most max_rows shapes (arrays of that length); *rows_out = shapes written. */
int32_t metasd_profile_shapes(metasd_ctx*, int32_t target_only, int32_t max_rows, int32_t* n_out, int32_t* k_out, int32_t* m_out,
                              double* ms_out, int64_t* launches_out, double* bytes_out, int32_t* rows_out);

/* ---- introspection ---------------------------------------------------------------------------- */

/* batch == 1: the row strides are those of gamma_max.  batch > 1: the buffers are packed for the gamma of
 * the last round - P [batch][gamma+1][V], Q [batch][gamma][V], BD and DRAFT [batch][gamma]. */
#define METASD_PEEK_P 0     /* float [gamma_max+1][V]  target logits of the last verify */
#define METASD_PEEK_Q 1     /* float [gamma_max][V]    drafter logits of the last draft */
#define METASD_PEEK_HIST 2  /* int32 [batch][max_ctx]  token history (committed + speculative) */
#define METASD_PEEK_BD 3    /* double [gamma_max]      sum_v min(p_j, q_j) of the last accept */
#define METASD_PEEK_FEAT 5  /* fp32 [max_ctx][d_model]   the target's features (contexts with feature_heads) */
#define METASD_PEEK_DRAFT 4 /* int32 [gamma_max + 1]   draft tokens d_1..d_gamma of the last draft; tree rounds: the token of every node (entry 0, the root, unused) */
/* Device pointer and byte size of an internal buffer (valid until metasd_destroy). */
int32_t metasd_peek(metasd_ctx*, int32_t what, void** dev_ptr_out, size_t* bytes_out);

/* Committed length l, number of positions in the KV cache of model (-1 target, k drafter),
 * rounds completed since the sequence's context was set.  Any pointer may be NULL. */
int32_t metasd_state(const metasd_ctx*, int32_t model, int32_t* l_out, int32_t* kv_len_out, int32_t* round_out);
/* The same for sequence seq of a batch (metasd_state reports sequence 0). */
int32_t metasd_state_seq(const metasd_ctx*, int32_t seq, int32_t model, int32_t* l_out, int32_t* kv_len_out,
                         int32_t* round_out);

/* How many accept steps of this context were taken a second time with one workgroup per position because the
 * workgroups that share a position did not meet within their bounded wait (see metasd_accept_logits; the
 * result is the same, the step is slower).  Expected to stay 0. */
int32_t metasd_accept_fallbacks(const metasd_ctx*, int64_t* count_out);

/* Message of the last error on this context (ctx == NULL: of the last context-free call on
 * this thread).  Never NULL. */
const char* metasd_last_error(const metasd_ctx*);

#ifdef __cplusplus
}
#endif
#endif /* METASD_H */
