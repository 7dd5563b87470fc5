/*
 * ver.h - C ABI of the VER learner step on one MI355X (gfx950).
 *
 * The library computes the learning phase of Variable Experience Rollout
 * (paper section 2.2) for a recurrent actor-critic trained with PPO:
 *
 *     ver_ingest           once per rollout, when the buffer comes in arrival
 *                          order (optional; the other calls take it bucketed)
 *     ver_gae              once per rollout
 *     ver_is_weight        once per rollout (optional)
 *     for every epoch, for every minibatch b:
 *         ver_pack_minibatch -> ver_lstm_fwd -> ver_ppo_loss -> ver_lstm_bwd
 *         -> ver_adam_step
 *
 * Conventions that hold for every entry point
 *  - "device" pointers are HIP device memory owned by the caller; "host"
 *    pointers are ordinary host memory.  The library never allocates, frees or
 *    keeps a pointer after the call returns, and never synchronises the
 *    stream: all work is enqueued on `stream` (a hipStream_t passed as void*,
 *    NULL = the default stream) and the call returns at once.
 *  - Scratch memory comes from a caller-provided device `workspace` of at
 *    least the size the matching *_workspace_bytes() query returns; its
 *    contents need not be initialised and are undefined afterwards, except
 *    that ver_lstm_bwd must be given the workspace ver_lstm_fwd filled.
 *  - Return value: VER_OK or a negative code.  Arguments are checked on the
 *    host only (null pointers, negative or inconsistent sizes); values that
 *    live in device memory (done flags, offsets) are not validated.
 *  - Rollout buffer layout (paper section 2.2: N environments contribute
 *    S = T x N steps in total, L_i >= 0 from environment i): flat step
 *    k = env_off[i] + t is step t of environment i; env_off[N+1] is the
 *    exclusive prefix sum of L, env_off[N] = S.  dones[k] = 1 means the
 *    episode ended WITH step k.
 *  - Packed layout (paper section 2.2, "Batching computation for learning",
 *    figure 2C): the M rows of a minibatch are time-major; timestep t holds
 *    batch_sizes[t] rows starting at row t_off[t]; row j of timestep t
 *    continues row j of timestep t-1 (pieces are ordered longest first).
 */
#ifndef VER_H
#define VER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    VER_OK = 0,
    VER_EINVAL = -1,       /* null pointer, negative size, b outside [0,B), B does not divide S ... */
    VER_EWORKSPACE = -2,   /* workspace missing or too small */
    VER_EUNSUPPORTED = -3, /* shape outside what the kernels handle (see each call) */
    VER_EHIP = -4,         /* a HIP call or kernel launch failed */
    VER_ETOOLARGE = -5     /* input above the stated maximum of an entry point with fixed scratch */
};

/* Text for a status code; never NULL.  Host only. */
const char* ver_status_string(int status);

/* ------------------------------------------------------------------------
 * ver_ingest - from the linear collection buffer to the ragged buffer.
 * Paper: section 2.2 "Batching computation for learning" (experience is
 * written into a linear buffer in GPU memory during collection) and section
 * 2.1 (inference workers store steps as they arrive: environments interleave,
 * each contributes a different number of steps).
 *
 * Slot a of the linear buffer holds a step of environment arr_env[a]; an
 * environment's own steps arrive in time order.  The call buckets the slots by
 * environment, arrival order kept inside a bucket (a stable sort):
 *   env_off[N+1]  exclusive prefix sum of the per-environment step counts
 *   order[S]      order[k] = arrival slot of flat step k of the ragged buffer
 *   info[4]       info[0] = steps that continue a stretch but whose counter
 *                 arr_t is not its predecessor's + 1 (0 when arr_t is NULL:
 *                 the counters are only checked, never used for ordering);
 *                 info[1] = slots whose id is outside [0, N): they are placed
 *                 behind all environments (env_off[N] = S - info[1]) and the
 *                 result must then not be used; info[2], info[3] = 0.
 * ver_ingest_gather then brings any per-step field into the new order:
 * dst row k = src row order[k], rows of row_bytes bytes (src != dst).
 * ver_ingest_dense is the closed form for equal-length rollouts stored
 * time-major (slot t*N + i = step t of environment i; the rollouts without
 * variable experience the paper compares against, section 5): env_off[i] = i*T,
 * order[i*T + t] = t*N + i.
 *
 * All pointers device: arr_env, arr_t (or NULL), order: int32[S]; env_off:
 * int32[N+1]; info: int32[4].  Outputs are bit-reproducible.  S = 0 is legal
 * (env_off all zero).  Errors: VER_EINVAL (N <= 0, negative sizes, null
 * pointers), VER_EUNSUPPORTED (S above 2^24), VER_EWORKSPACE.
 */
size_t ver_ingest_workspace_bytes(int32_t N, int32_t S);
int ver_ingest(const int32_t* arr_env, const int32_t* arr_t, int32_t N, int32_t S,
               int32_t* env_off, int32_t* order, int32_t* info,
               void* workspace, size_t workspace_bytes, void* stream);
int ver_ingest_dense(int32_t T, int32_t N, int32_t* env_off, int32_t* order, void* stream);
int ver_ingest_gather(const int32_t* order, int32_t S, const void* src, int32_t row_bytes,
                      void* dst, void* stream);
/* The same for several fields in one launch (a rollout has a dozen per-step
 * fields, each a few microseconds of work at the paper's sizes): field f moves
 * dst[f] row k = src[f] row order[k], rows of row_bytes[f] bytes.  src, dst and
 * row_bytes are HOST arrays of n_fields entries (device pointers inside), read
 * before the call returns; n_fields <= VER_INGEST_MAX_FIELDS, else VER_EINVAL. */
#define VER_INGEST_MAX_FIELDS 24
int ver_ingest_gather_batch(const int32_t* order, int32_t S, int32_t n_fields,
                            const void* const* src, const int32_t* row_bytes,
                            void* const* dst, void* stream);

/* ------------------------------------------------------------------------
 * ver_gae - advantages and value targets over the ragged buffer.
 * Paper: section 4 "Training" (PPO with Generalized Advantage Estimation),
 * hyper-parameter table (gamma 0.99, lambda 0.95); ragged stretches and
 * episode ends inside them from section 2.2 / figure 2B.
 *
 * Per environment i, backwards over its stretch, with nd = 1 - dones[k]:
 *     delta_k = rewards[k] + gamma * nd * V_next - values[k]
 *     adv[k]  = delta_k + gamma * lambda * nd * adv_next
 *     ret[k]  = adv[k] + values[k]
 * where V_next / adv_next are values[k+1] / adv[k+1] inside the stretch and
 * last_values[i] / 0 after its last step.  No normalisation.
 *
 * All pointers device.  rewards, values, adv, ret: float[S]; dones: uint8[S];
 * last_values: float[N]; env_off: int32[N+1].  S = 0 is legal (no work).
 * Output is deterministic (no atomics on floats).  Any alignment is accepted;
 * 16-byte aligned rewards, values, adv, ret (4-byte aligned dones) take
 * 16-byte accesses.
 * The scan is a single pass in which tiles of 2048 steps wait (bounded) for
 * what the tiles after them publish.  Should such a wait ever give up (it
 * cannot while the GPU makes progress), workspace word 1 (int32) is non-zero
 * once the stream has drained and the outputs of that tile, and of the tiles
 * towards the start of the buffer that depend on it, are NaN: never a
 * plausible wrong number.
 */
size_t ver_gae_workspace_bytes(int32_t S);
int ver_gae(const float* rewards, const float* values, const uint8_t* dones,
            const float* last_values, const int32_t* env_off, int32_t N, int32_t S,
            float gamma, float lambda, float* adv, float* ret,
            void* workspace, size_t workspace_bytes, void* stream);

/*
 * ver_gae_static - ver_gae for callers that cannot allocate device memory or
 * have none to hand over as a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * kernels as ver_gae, without the workspace: the scan's scratch (ticket, error
 * word, three 64-bit words per tile of 2048 steps) lives in a device array of
 * fixed size inside the library, 48.25 KiB that every GPU the library is used
 * on holds until the process ends.  The call allocates and frees nothing; the
 * first call on a device looks the array's address up (once per device, with
 * that device current).
 * Limit: S <= VER_GAE_STATIC_MAX_STEPS, otherwise VER_ETOOLARGE and nothing is
 * enqueued (the largest rollout of the paper's configurations has 32768 steps).
 * Every call on a GPU uses that GPU's one array: the part a call uses is
 * cleared on the stream before its kernel starts, so calls one after the other
 * on a stream need nothing from the caller, but two calls of one process that
 * may overlap in time on the same GPU (issued on different streams) race on it
 * and must be ordered by the caller.  Another process has its own copy.
 * The error word of ver_gae's workspace has no counterpart that the caller
 * can read here: a wait that gave up shows as NaN outputs only.
 */
#define VER_GAE_STATIC_MAX_STEPS (1 << 22)
int ver_gae_static(const float* rewards, const float* values, const uint8_t* dones,
                   const float* last_values, const int32_t* env_off, int32_t N, int32_t S,
                   float gamma, float lambda, float* adv, float* ret, void* stream);

/* ------------------------------------------------------------------------
 * ver_is_weight - truncated importance weight of every step of the buffer.
 * Paper: section 4 "Training" (experience from fast environments is
 * over-represented under variable experience rollouts; corrected with
 * truncated importance sampling) and the appendix hyper-parameter table
 * (importance sampling on, maximum weight 1.0).  The paper gives no formula;
 * reading implemented: every step of environment i carries
 *     w_i = min(max_is, (S / N) / L_i),   L_i = env_off[i+1] - env_off[i],
 * the share an environment would have under equal-length rollouts over the
 * share it has; constant inside a stretch.  The weights feed ver_ppo_loss
 * (is_weight) after ver_pack_minibatch has gathered them into packed order.
 *
 * env_off: device int32[N+1]; weight: device float[S], 16-byte aligned.  The quotient is
 * formed in double and rounded once.  max_is <= 0 or N <= 0 is VER_EINVAL;
 * S = 0 is legal (no work).  The weight array is also the call's scratch:
 * from 2^20 steps on a first kernel leaves environment indices in it, which
 * the second overwrites with the weights, so its contents are only meaningful
 * once the call's work on the stream has finished.
 */
int ver_is_weight(const int32_t* env_off, int32_t N, int32_t S, float max_is,
                  float* weight, void* stream);

/* ------------------------------------------------------------------------
 * ver_pack_minibatch - VER minibatch creation + packed-sequence layout.
 * Paper: section 2.2 "Learning mini-batch creation" (sequences start at a
 * stretch start or after an episode end; randomly ordered; the first S/B
 * steps form minibatch 0, the next S/B minibatch 1, ...) and "Batching
 * computation for learning" (all elements of a timestep contiguous).
 *
 * Rule implemented (the parts the paper leaves open are fixed as follows):
 *  1. sequences are discovered in (environment, time) order; that order is
 *     the sequence id;
 *  2. random order = ascending (seq_key[first step of the sequence], id);
 *     seq_key holds one caller-drawn 32-bit key per step, only keys at
 *     sequence heads are read;
 *  3. the sequences laid end to end form a stream of S steps; minibatch b
 *     is stream positions [b*M, (b+1)*M), M = S/B; a sequence crossing a
 *     cut is split, the tail piece is not an episode start;
 *  4. pieces of the minibatch are ordered longest first, ties by stream
 *     position;
 *  5. a piece is an episode start if it begins right after a done step, or
 *     begins a stretch whose env_started_episode[i] is non-zero.
 *
 * Index outputs (device, caller sizes them for the upper bound M):
 *   info[4]            n_seq, T_max, K (sequences in the whole buffer), 0
 *   seq_first[M]       flat step of each piece's first step
 *   seq_len[M]         piece lengths (non-increasing)
 *   seq_is_ep_start[M] uint8
 *   batch_sizes[M]     rows per timestep (entries >= T_max are zero)
 *   t_off[M+1]         exclusive prefix sum of batch_sizes (entries > T_max = M)
 *   gather_idx[M]      packed row -> flat step
 * Only the first n_seq (resp. T_max) entries carry pieces (timesteps).
 *
 * Optional gathers, each skipped when its source or destination is NULL:
 *   obs[S,D] float        -> obs_packed[M,D]  float, or bf16 when obs_packed_bf16 != 0
 *   actions[S,act_bytes]  -> actions_packed[M,act_bytes]   (raw bytes per step)
 *   logp_old/adv/ret/is_weight[S] -> *_packed[M]
 *   rnn_h/rnn_c[n_layers,S,H] (state each layer had BEFORE step k at
 *   collection time) -> h0/c0[n_layers,seq_cap,H]: row j = state of piece j's
 *   first step, zeros if the piece is an episode start.  seq_cap >= n_seq
 *   must hold (M always suffices); rows >= n_seq are left untouched.
 *
 * Errors: VER_EINVAL if B <= 0, b outside [0,B), B does not divide S, or a
 * required pointer is NULL.  Integer outputs are bit-reproducible.
 */
typedef struct {
    /* rollout buffer */
    const uint8_t* dones;               /* [S] */
    const int32_t* env_off;             /* [N+1] */
    const uint8_t* env_started_episode; /* [N] or NULL (= all 0) */
    const uint32_t* seq_key;            /* [S] */
    int32_t N, S, B, b;
    /* index outputs */
    int32_t* info;
    int32_t* seq_first;
    int32_t* seq_len;
    uint8_t* seq_is_ep_start;
    int32_t* batch_sizes;
    int32_t* t_off;
    int32_t* gather_idx;
    /* optional gathers */
    const float* obs;
    int32_t D;
    void* obs_packed;
    int32_t obs_packed_bf16;
    const void* actions;
    int32_t act_bytes;
    void* actions_packed;
    const float* logp_old;
    const float* adv;
    const float* ret;
    const float* is_weight;
    float* logp_old_packed;
    float* adv_packed;
    float* ret_packed;
    float* is_weight_packed;
    const float* rnn_h;
    const float* rnn_c;
    int32_t n_layers, H, seq_cap;
    float* h0;
    float* c0;
    /* scratch */
    void* workspace;
    size_t workspace_bytes;
    /* non-zero: the index outputs already hold this minibatch's values (written by ver_pack_index_batch
     * or by an earlier call with the same rollout, keys, B and b): only the gathers are performed */
    int32_t index_ready;
} ver_pack_args;

size_t ver_pack_workspace_bytes(int32_t N, int32_t S, int32_t B);
int ver_pack_minibatch(const ver_pack_args* args /* host */, void* stream);

/*
 * ver_pack_index_batch - the index outputs of n minibatches in one launch.
 * The minibatches of an update (every epoch's keys, every b) depend only on the
 * rollout, never on the weights, and each takes one workgroup: args is a host
 * array of n argument blocks that share dones, env_off, env_started_episode,
 * N, S and B and differ in seq_key, b, the index outputs and the workspace
 * (each block its own: VER_EINVAL if two share info or workspace).  Writes
 * info .. t_off of every block exactly as ver_pack_minibatch would; gather
 * fields and gather_idx are ignored.  A later ver_pack_minibatch with
 * index_ready != 0 on the same block performs the gathers (and gather_idx).
 */
int ver_pack_index_batch(const ver_pack_args* args /* host array */, int32_t n, void* stream);

/* ------------------------------------------------------------------------
 * ver_lstm_fwd / ver_lstm_bwd - multi-layer LSTM actor-critic over a packed
 * minibatch, and back-propagation through time.
 * Paper: section 4 "Architecture" and section 3 (embedding joined with the
 * state vector -> 2-layer LSTM -> action distribution and value); sequences
 * for back-propagation through time from section 2.2.
 *
 * Cell (gate order i, f, g, o; two bias vectors; no peepholes/projection):
 *     z = W_ih x_t + b_ih + W_hh h_{t-1} + b_hh
 *     c_t = sigm(z_f) * c_{t-1} + sigm(z_i) * tanh(z_g);  h_t = sigm(z_o) * tanh(c_t)
 * Layer l+1 reads h_t of layer l.  Heads on the top layer:
 *     head_out = W_a h + b_a  [act_dim],   value = w_v . h + b_v.
 *
 * cfg.compute: 0 = all contractions in fp32 (fp32 MFMA); 1 = operands of the
 * contractions rounded to bf16 (round to nearest even), accumulation, biases,
 * gate non-linearities, cell state, saved activations and all outputs fp32.
 * cfg.x_bf16: x_packed holds bf16 (only with compute = 1) instead of float.
 *
 * weights (host array of 4*n_layers + 4 device pointers, all float):
 *   per layer l: W_ih[4H, D_l], W_hh[4H, H], b_ih[4H], b_hh[4H]  (D_0 = input_dim, D_l = H)
 *   then W_a[act_dim, H], b_a[act_dim], w_v[H], b_v[1].
 * weight_grads: same order and shapes; OVERWRITTEN with the gradient of the
 * minibatch loss (not accumulated).
 *
 * info, batch_sizes, t_off: as written by ver_pack_minibatch (device; the
 * kernels read n_seq and T_max from info on the device, so no host round trip
 * is needed between pack and the LSTM).  h0, c0: float[n_layers, seq_cap, H]
 * initial state per piece, or NULL for zeros.
 * head_out: float[M, act_dim]; value: float[M].
 * ver_lstm_bwd: d_head_out[M, act_dim], d_value[M] are the loss gradients
 * (e.g. from ver_ppo_loss); d_x: float[M, input_dim] or NULL.  It must be
 * called with the same cfg, M, metadata, x_packed, h0/c0, weights and
 * workspace as the forward call it differentiates.
 *
 * Errors: VER_EUNSUPPORTED unless hidden is a multiple of 64 with
 * 64 <= hidden <= 1024 (compute = 1) or <= 512 (compute = 0) - a wave keeps
 * its share of W_hh in registers and 16 rows of gate gradients in LDS -,
 * input_dim a multiple of 4, 1 <= n_layers <= 8, 1 <= act_dim <= 63, and
 * M * hidden < 2^27 (32-bit byte offsets inside an activation array).
 * workspace word 0 (int32) is non-zero after the stream has drained if a
 * device-side wait timed out (should never happen; results are then
 * undefined).  Outputs are deterministic.
 *
 * The time loops run as persistent kernels that need the whole GPU (one
 * workgroup on every CU at the same time, cooperating per XCD): kernels of
 * other streams or processes that hold CUs for long can make their bounded
 * waits time out.  ver_lstm_fwd / ver_lstm_bwd return VER_EUNSUPPORTED on a
 * device that is not a whole MI355X (gfx950 with 256 compute units; the
 * device is queried once).  Networks of two layers run both layers' time
 * loops in one launch; cfg.layer_by_layer = 1 makes them run layer by layer
 * like any other depth - a diagnostic switch, results agree up to the order
 * of fp32 additions (forward and backward must be called with the same value).
 */
typedef struct {
    int32_t n_layers;
    int32_t input_dim;
    int32_t hidden;
    int32_t act_dim;
    int32_t compute;
    int32_t x_bf16;
    int32_t layer_by_layer;   /* 0 (default) or 1, see above */
} ver_lstm_cfg;

size_t ver_lstm_workspace_bytes(const ver_lstm_cfg* cfg, int32_t M);
int ver_lstm_fwd(const ver_lstm_cfg* cfg, const void* x_packed, int32_t M,
                 const int32_t* info, const int32_t* batch_sizes, const int32_t* t_off,
                 const float* h0, const float* c0, int32_t seq_cap,
                 const float* const* weights /* host array */,
                 float* head_out, float* value,
                 void* workspace, size_t workspace_bytes, void* stream);
int ver_lstm_bwd(const ver_lstm_cfg* cfg, const void* x_packed, int32_t M,
                 const int32_t* info, const int32_t* batch_sizes, const int32_t* t_off,
                 const float* h0, const float* c0, int32_t seq_cap,
                 const float* const* weights /* host array */,
                 const float* d_head_out, const float* d_value,
                 float* const* weight_grads /* host array */, float* d_x,
                 void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * ver_ppo_loss - fused PPO loss and its gradient w.r.t. the heads' outputs.
 * Paper: section 2.2 "Learning method" (PPO); hyper-parameter table: clip
 * 0.2, value coefficient 0.5, no clipped value loss, no advantage
 * normalisation; fixed entropy coefficient 1e-4 for benchmarks (appendix,
 * "Hyperparamaters"); categorical or independent-Gaussian actions
 * (section 4 "Architecture").
 *
 * Per packed row p (w_p = is_weight[p], 1 when is_weight is NULL):
 *   categorical (dist 0): logp = head_out[p, a_p] - logsumexp(head_out[p, :]),
 *       entropy of softmax(head_out[p, :]); actions int32[M]
 *   Gaussian (dist 1): mean = head_out[p, :], std = exp(log_std), independent
 *       dims; actions float[M, act_dim]
 *   rho = exp(logp - logp_old[p])
 *   l_pi = -min(rho * adv, clamp(rho, 1-clip, 1+clip) * adv);  l_v = 0.5 * (value - ret)^2
 * total = mean(w l_pi) + value_coef * mean(w l_v) - entropy_coef * mean(w entropy),
 * means over the M rows.  The gradient through min/clamp follows the selected
 * branch; the unclipped branch wins ties.
 *
 * scalars (device float[6]): total, policy, value, entropy (mean),
 * approx_kl = mean(logp_old - logp), clip_frac = mean(|rho - 1| > clip).
 * d_head_out[M, act_dim], d_value[M], d_log_std[act_dim] (Gaussian only, may
 * be NULL for categorical): gradient of total.  Reductions are done in a
 * fixed order: results are bit-reproducible.  M = 0 is VER_EINVAL.
 */
typedef struct {
    float clip;
    float value_coef;
    float entropy_coef;
    int32_t dist;     /* 0 categorical, 1 diagonal Gaussian */
    int32_t act_dim;  /* 1..63 */
} ver_ppo_cfg;

size_t ver_ppo_loss_workspace_bytes(int32_t M, int32_t act_dim);
int ver_ppo_loss(const ver_ppo_cfg* cfg, int32_t M,
                 const float* head_out, const float* value, const float* log_std,
                 const void* actions_packed, const float* logp_old, const float* adv,
                 const float* ret, const float* is_weight,
                 float* scalars, float* d_head_out, float* d_value, float* d_log_std,
                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * ver_ppo_loss_learned_entropy - the same loss with the learned entropy
 * coefficient of the training runs in place of the fixed one.
 * Paper: section 4 "Training" (minimum-entropy constraint with a learned
 * coefficient: alpha * (lambda - sg[H]) - sg[alpha] * H, sg = stop gradient,
 * target entropy lambda = 0); appendix hyper-parameter table (initial
 * coefficient 1e-3, bounds [1e-4, 1.0]).
 *
 * alpha: device float[1], read only: the current coefficient.  H is the
 * (weighted) mean entropy over the M rows, the number scalars[3] reports.
 *   total = mean(w l_pi) + value_coef * mean(w l_v) + alpha * (target_entropy - H) - alpha * H
 * The policy is given the gradient of - alpha * H with alpha constant, i.e.
 * d_head_out, d_value and d_log_std are those of ver_ppo_loss at
 * entropy_coef = alpha (cfg->entropy_coef is ignored).
 * d_alpha: device float[1], receives alpha_sign * (target_entropy - H), the
 * derivative of the expression w.r.t. alpha with H constant.  alpha_sign = +1
 * is the expression as printed; -1 gives a descending optimiser the ascent
 * direction of the constraint's multiplier (printed as a minimisation, alpha
 * shrinks while the entropy is below the target).  Other values: VER_EINVAL.
 * Keeping alpha inside its bounds is the optimiser's part
 * (ver_adam_step_bounded).  Everything else as ver_ppo_loss.
 */
int ver_ppo_loss_learned_entropy(const ver_ppo_cfg* cfg, int32_t M,
                                 const float* head_out, const float* value, const float* log_std,
                                 const void* actions_packed, const float* logp_old, const float* adv,
                                 const float* ret, const float* is_weight,
                                 const float* alpha, float target_entropy, float alpha_sign,
                                 float* scalars, float* d_head_out, float* d_value, float* d_log_std,
                                 float* d_alpha, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * ver_adam_step - the optimiser step that follows ver_lstm_bwd.
 * Paper: section 4 "Training" and the appendix hyper-parameter table: Adam,
 * initial learning rate 2.5e-4 decayed to zero with a cosine schedule.  The
 * optimiser is only cited: this is the bias-corrected step of the cited Adam
 * paper,
 *   m <- beta1 m + (1-beta1) g,  v <- beta2 v + (1-beta2) g^2,
 *   p <- p - lr_k * (m / (1-beta1^t)) / (sqrt(v / (1-beta2^t)) + eps),  t = k+1,
 * with lr_k = lr_final + (lr0 - lr_final) * (1 + cos(pi * min(k, total_steps)
 * / total_steps)) / 2 for the k-th step counted from 0.  Readings where the
 * paper is silent: beta1 0.9, beta2 0.999, eps 1e-8 are the caller's to set
 * (defaults of the cited paper); no weight decay; gradient clipping is
 * optional, by the global 2-norm over all tensors of the call:
 * g <- g * min(1, max_grad_norm / (norm + 1e-6)), off when max_grad_norm <= 0.
 *
 * params, grads, exp_avg, exp_avg_sq: host arrays of n_tensors device
 * pointers (float, 16-byte aligned; grads are read only, the other three are
 * updated in place); sizes: host array of element counts (may be 0).
 * n_tensors <= VER_ADAM_MAX_TENSORS.  step_index = k (0 for the first step).
 * grad_norm: device float[1] that receives the global 2-norm of the gradients
 * before clipping, or NULL (only allowed without clipping).  All tensors are
 * handled by one launch (28 bytes of HBM traffic per parameter); the norm, when
 * asked for, by a deterministic two-stage reduction before it.
 * Errors: VER_EINVAL (null pointers, negative sizes, total_steps <= 0,
 * n_tensors out of range, clipping without grad_norm), VER_EWORKSPACE.
 */
#define VER_ADAM_MAX_TENSORS 48
typedef struct {
    float lr0;            /* initial learning rate (paper: 2.5e-4) */
    float lr_final;       /* final learning rate (paper: 0) */
    int64_t total_steps;  /* optimiser steps over which the cosine runs */
    float beta1, beta2, eps;
    float max_grad_norm;  /* <= 0: no clipping */
} ver_adam_cfg;

size_t ver_adam_workspace_bytes(void);
int ver_adam_step(const ver_adam_cfg* cfg, int32_t n_tensors, float* const* params, const float* const* grads,
                  float* const* exp_avg, float* const* exp_avg_sq, const int64_t* sizes, int64_t step_index,
                  float* grad_norm, void* workspace, size_t workspace_bytes, void* stream);

/*
 * ver_adam_step_bounded - the same step followed by a projection of every
 * tensor onto a box: p <- min(max(p, lower[i]), upper[i]) for all elements of
 * tensor i.  Paper: the learned entropy coefficient is kept inside bounds
 * (appendix hyper-parameter table: [1e-4, 1.0]); the projection after the step
 * is our reading of how.  lower, upper: host float arrays of n_tensors entries
 * (-INFINITY / INFINITY = unbounded), either may be NULL (= unbounded for all).
 * lower[i] > upper[i] or a NaN bound is VER_EINVAL.  Everything else as
 * ver_adam_step, which is this call with both arrays NULL.
 */
int ver_adam_step_bounded(const ver_adam_cfg* cfg, int32_t n_tensors, float* const* params, const float* const* grads,
                          float* const* exp_avg, float* const* exp_avg_sq, const int64_t* sizes,
                          const float* lower, const float* upper, int64_t step_index,
                          float* grad_norm, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Kernel timing for benchmarks (measurement plumbing, not part of the method).
 * While enabled, the library brackets the kernels of the selected classes with
 * HIP events on the stream of the call.  ver_profile_read waits for the
 * recorded events, adds the elapsed time and launch count of every class into
 * total_ms / launches (host arrays of VER_PROF_COUNT entries, overwritten) and
 * forgets the events.  mask: bit i enables class i.  Not thread safe.
 */
enum {
    VER_PROF_GAE = 0,
    VER_PROF_PACK_INDEX = 1,
    VER_PROF_PACK_GATHER = 2,
    VER_PROF_LSTM_PREP = 3,
    VER_PROF_LSTM_GEMM_FWD = 4,
    VER_PROF_LSTM_REC_FWD = 5,
    VER_PROF_HEADS_FWD = 6,
    VER_PROF_LOSS = 7,
    VER_PROF_HEADS_BWD = 8,
    VER_PROF_LSTM_REC_BWD = 9,
    VER_PROF_LSTM_GEMM_DX = 10,
    VER_PROF_LSTM_GEMM_DW = 11,
    VER_PROF_LSTM_DBIAS = 12,
    VER_PROF_ADAM = 13,
    VER_PROF_IS_WEIGHT = 14,
    VER_PROF_INGEST = 15,
    VER_PROF_COUNT = 16
};
int ver_profile_enable(uint32_t mask);
int ver_profile_read(double* total_ms, int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* VER_H */
