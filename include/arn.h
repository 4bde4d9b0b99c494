/*
 * arn -- Accelerated-RL Network: the neural-network hot path of Stooke & Abbeel,
 * "Accelerated Methods for Deep Reinforcement Learning", as hand-written gfx950
 * (MI355X) kernels behind a C ABI.
 *
 * The network is the Atari "Nature" CNN that the paper's appendix "Atari Frame
 * Processing" calls the standard 3-convolutional-layer network:
 *   uint8 [4,84,84] -> /255 -> conv 8x8/4 x32 -> conv 4x4/2 x64 -> conv 3x3/1 x64
 *   -> fc 3136->512 (ReLU after every hidden layer) -> heads.
 * With geometry ARN_GEOM_PAPER the same layers take the frame size and padding the
 * appendix states for the paper's own runs: uint8 [4,104,80], no padding on conv1,
 * padding 1 on conv2 and conv3, feature maps 25x19 -> 12x9 -> 12x9, fc 6912->512.
 * Heads: policy logits [A] + value [1]   (head_kind ARN_HEAD_PV),
 *        categorical atom logits [A,51]   (head_kind ARN_HEAD_C51),
 *        scalar action values Q [A]       (head_kind ARN_HEAD_Q), or
 *        advantages [A] + state value [1] combined as Q = V + A - mean(A)
 *                                         (head_kind ARN_HEAD_DUEL; one shared hidden layer).
 *
 * Two operations follow the paper's problem statement:
 *   - batched action-selection inference: one forward over all simulators'
 *     observations per environment step (section "Synchronized Sampling");
 *   - the local gradient of a training batch, step 1 of the synchronous
 *     data-parallel update (section "Synchronous Multi-GPU Optimization"), for
 *     the advantage actor-critic, PPO clipped-surrogate, Categorical-DQN and
 *     DQN (optionally Double-DQN) objectives (section "RL Algorithm Background").
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers owned by the caller and must be
 *     16-byte aligned (256-byte for workspace and packed weights).  `arn_config`
 *     and `arn_batch` structs themselves live in HOST memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work and return; they never synchronise, allocate or free
 *     device memory.  arn_train_step_grads also uses one library-owned stream
 *     per device (created on first use, default priority) for work that can run
 *     next to the caller's stream; it is forked from and joined back to `stream`
 *     with events inside the call, so to the caller the call behaves as if all
 *     of its work were on `stream`.  Set ARN_SINGLE_STREAM=1 to disable it.
 *     That stream and its events are shared by all calls on a device: two
 *     arn_train_step_grads calls issued concurrently from different host threads
 *     on the same device are not supported (issue them from one thread, on one
 *     or several streams; successive calls are ordered by the events).  The
 *     profiling switch (arn_profile_*) is likewise process-global.
 *   - Return value: ARN_OK (0) or a negative arn_status.  Argument errors are
 *     detected on the host before anything is launched.
 *   - Arithmetic: bf16 MFMA operands, fp32 accumulation, fp32 epilogues and
 *     losses.  Gradients are reduced over the batch in a fixed order, so
 *     repeated calls on the same inputs give bit-identical results.
 *
 * Flat fp32 parameter / gradient vector, canonical order (row-major tensors):
 *   conv1.W[32,4,8,8] conv1.b[32] conv2.W[64,32,4,4] conv2.b[64]
 *   conv3.W[64,64,3,3] conv3.b[64] fc.W[512,3136] fc.b[512]
 *   (fc input index = c*49 + y*7 + x; ARN_GEOM_PAPER: fc.W[512,6912], index c*108 + y*9 + x), then
 *   PV : pi.W[A,512] pi.b[A] v.W[1,512] v.b[1]
 *   C51: c51.W[A*atoms,512] (row a*atoms+j) c51.b[A*atoms]
 *   Q  : q.W[A,512] q.b[A]
 *   DUEL: adv.W[A,512] adv.b[A] val.W[1,512] val.b[1]        (same shape as PV)
 * ARN_GEOM_A3C: conv1.W[16,4,8,8] conv1.b[16] conv2.W[32,16,4,4] conv2.b[32] fc.W[256,3456] (input index
 *   c*108 + y*9 + x) fc.b[256], then the heads as above with 256 in place of 512.  This network runs on the
 *   kernels of the 104x80 three-convolution network, embedded in it with zero filters and an identity third
 *   layer (exact: the embedded network computes the same function and the same gradients); it is supported for
 *   completeness of the paper's networks, not tuned.
 */
#ifndef ARN_H
#define ARN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ARN_OK = 0,
    ARN_EINVAL = -1,     /* null or misaligned pointer, B <= 0 or B > 2^20 (1,048,576 samples per call) */
    ARN_ESHAPE = -2,     /* unsupported num_actions / num_atoms / head for this call */
    ARN_EKIND = -3,      /* unknown head_kind / loss_kind / mode */
    ARN_EWORKSPACE = -4, /* workspace smaller than arn_workspace_bytes() */
    ARN_EARCH = -5,      /* current device is not gfx950 */
    ARN_EHIP = -6,       /* a HIP runtime call or launch failed */
    ARN_ESTATIC = -7     /* arn_policy_forward_static: the call needs more scratch memory than ARN_STATIC_SCRATCH_BYTES */
} arn_status;

enum { ARN_HEAD_PV = 0, ARN_HEAD_C51 = 1, ARN_HEAD_Q = 2, ARN_HEAD_DUEL = 3 };
enum { ARN_LOSS_A2C = 0, ARN_LOSS_PPO = 1, ARN_LOSS_C51 = 2, ARN_LOSS_DQN = 3 };
enum { ARN_MODE_FORWARD = 0, ARN_MODE_TRAIN = 1 };
/* frame size and padding of the convolution stack (appendix "Atari Frame Processing") */
enum { ARN_GEOM_84 = 0,      /* 84x84 frames, no padding: 20x20 -> 9x9 -> 7x7, fc input 3136 */
       ARN_GEOM_PAPER = 1,   /* 104x80 frames, padding 1 on conv2/conv3: 25x19 -> 12x9 -> 12x9, fc input 6912 */
       ARN_GEOM_A3C = 2 };   /* the 2-convolution policy-gradient network of the same appendix on 104x80 frames:
                                conv 8x8/4 x16 -> conv 4x4/2 x32 (padding 1) -> fc 3456 -> 256; maps 25x19 -> 12x9.
                                (Filter counts: those of the publication the appendix cites for this network.) */

typedef struct {
    int32_t num_actions;   /* 1..31 for PV, Q, DUEL; 1..18 for C51 */
    int32_t head_kind;     /* ARN_HEAD_PV, ARN_HEAD_C51, ARN_HEAD_Q or ARN_HEAD_DUEL */
    int32_t num_atoms;     /* C51 only: 2..64 (51 in the paper's Categorical DQN) */
    float v_min, v_max;    /* C51 support end points (-10, 10) */
    float gamma;           /* C51 and DQN discount (0.99) */
    float clip_eps;        /* PPO clip range (0.1) */
    float value_coef;      /* weight of mean((V-ret)^2) (0.5) */
    float entropy_coef;    /* weight of the mean-entropy bonus (0.01) */
    int32_t double_q;      /* DQN: 1 = the online network picks the next action (Double-DQN), 0 = the target network */
    int32_t geometry;      /* ARN_GEOM_84 (0), ARN_GEOM_PAPER or ARN_GEOM_A3C; anything else is ARN_ESHAPE */
} arn_config;

/* Number of fp32 entries of the flat parameter vector; 0 on a bad config. */
size_t arn_param_count(const arn_config *cfg);

/* Bytes of the packed (bf16, kernel-layout) copy of the parameters that
 * arn_weights_prepare writes; 0 on a bad config.  It holds forward-layout and
 * input-gradient-layout copies of every weight matrix plus fp32 biases. */
size_t arn_packed_bytes(const arn_config *cfg);

/* Bytes of scratch device memory that a call with batch size B needs.
 * mode = ARN_MODE_FORWARD (arn_policy_forward) or ARN_MODE_TRAIN
 * (arn_train_step_grads).  0 on bad arguments. */
size_t arn_workspace_bytes(const arn_config *cfg, int B, int mode);

/* Convert the flat fp32 parameters to the packed form.  Belongs to the
 * parameter update (step 3 of the synchronous procedure), not to the gradient
 * step; call it once per update.  w_fp32: [arn_param_count], device.
 * w_packed: [arn_packed_bytes], device, overwritten. */
int arn_weights_prepare(const arn_config *cfg, const float *w_fp32, void *w_packed, void *stream);

/* Batched action-selection inference (section "Synchronized Sampling").
 *   obs    : uint8 [B,4,84,84] (NCHW; [B,4,104,80] with ARN_GEOM_PAPER and ARN_GEOM_A3C), read only
 *   logits : PV: fp32 [B,A]; C51: fp32 [B,A,atoms]; Q, DUEL: the action values Q [B,A].  Required.
 *   value  : PV: fp32 [B], required.  C51: expected action values Q [B,A], or NULL.
 *            Q, DUEL: max_a Q [B], required.
 *   probs  : PV: softmax over actions [B,A]; C51: softmax over atoms [B,A,atoms]; or NULL.
 *            Must be NULL for Q and DUEL (ARN_ESHAPE otherwise).
 *   greedy : int32 [B] -- lowest-index argmax of the logits (PV) or of Q (C51, Q, DUEL); or NULL
 * Outputs are overwritten.  Workspace contents are undefined afterwards. */
int arn_policy_forward(const arn_config *cfg, const void *w_packed, const uint8_t *obs, int B,
                       float *logits, float *value, float *probs, int32_t *greedy,
                       void *workspace, size_t workspace_bytes, void *stream);

/* arn_policy_forward for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, outputs and kernels as
 * arn_policy_forward, but the scratch memory is a buffer of ARN_STATIC_SCRATCH_BYTES that is part of the
 * library's device image (one copy per GPU, held until the process ends); the call allocates and frees nothing.
 *   - Accepted iff arn_workspace_bytes(cfg, B, ARN_MODE_FORWARD) <= ARN_STATIC_SCRATCH_BYTES (for example every
 *     policy/value, Q or dueling head on 84x84 frames up to B = 256); otherwise ARN_ESTATIC and nothing is launched.
 *   - All calls on one GPU share that buffer and it keeps the last call's contents (every call rewrites what it
 *     reads): calls that overlap in time on one GPU -- from two streams or two host threads -- race; order them
 *     on one stream or with events.
 *   - The first call on a device looks the buffer's address up (hipGetSymbolAddress); make that call outside
 *     graph capture. */
#define ARN_STATIC_SCRATCH_BYTES (32u << 20)
int arn_policy_forward_static(const arn_config *cfg, const void *w_packed, const uint8_t *obs, int B,
                              float *logits, float *value, float *probs, int32_t *greedy, void *stream);

/* Inference that returns actions, as the paper's sampler does (section "Synchronized Sampling": the
 * simulator processes receive actions, not logits).  The random numbers are inputs:
 *   u, u2  : fp32 [B], uniform in [0,1)
 *   PV     : categorical draw by inverse CDF -- the first action whose cumulative probability exceeds
 *            u (the last action if rounding leaves the total below u); u2 and epsilon are ignored.
 *   C51, Q, DUEL: epsilon-greedy -- u < epsilon takes action floor(u2*A), otherwise the greedy action.
 *   action : int32 [B], overwritten.  Required.
 *   logp   : PV: fp32 [B] log pi(action) (what PPO later needs as old_logp), or NULL; must be NULL otherwise.
 * Same workspace as arn_policy_forward (ARN_MODE_FORWARD). */
int arn_policy_act(const arn_config *cfg, const void *w_packed, const uint8_t *obs, int B, const float *u,
                   const float *u2, float epsilon, int32_t *action, float *logp, void *workspace,
                   size_t workspace_bytes, void *stream);

typedef struct {
    const uint8_t *obs;        /* [B,4,84,84] ([B,4,104,80] with ARN_GEOM_PAPER) */
    const int32_t *action;     /* [B], 0 <= a < A (values outside are clamped into range, not reported) */
    const float *adv;          /* [B]  a2c, ppo: advantage estimates (constants) */
    const float *ret;          /* [B]  a2c, ppo: value regression targets */
    const float *old_logp;     /* [B]  ppo: log pi_old(a|s) */
    const uint8_t *next_obs;   /* same shape as obs;  c51, dqn */
    const float *reward;       /* [B]  c51, dqn */
    const uint8_t *done;       /* [B]  c51, dqn: 1 = terminal transition */
    const void *w_target_packed; /* c51, dqn: packed target-network parameters */
    int32_t *next_action;      /* [B]  c51, dqn: OUTPUT, or NULL: the greedy next action a* the step bootstrapped from
                                  (overwritten; 16-byte aligned) */
} arn_batch;

/* Local gradient of one training batch (step 1 of section "Synchronous
 * Multi-GPU Optimization").  Every loss term is a mean over the batch:
 *   a2c: -mean(log pi(a) adv) + value_coef mean((V-ret)^2) - entropy_coef mean(H)
 *   ppo: -mean(min(rho adv, clip(rho,1-eps,1+eps) adv)) + same value/entropy terms,
 *        rho = exp(log pi(a) - old_logp)
 *   c51: -mean(sum_i m_i log p_i(s,a)), m = projection onto the support of the
 *        target network's distribution for its greedy next action, shifted by
 *        reward and gamma (1-done).
 *   dqn: mean((y - Q(s,a))^2), y = reward + gamma (1-done) Q(s', a*; target network), a* = the greedy
 *        action of the target network on s', or of the online network when cfg->double_q is set
 *        (one more forward pass); y is a constant.
 *   The passes that carry no gradient -- the target network's forward on next_obs and Double-DQN's selection
 *   forward -- run one fp16 product per layer, as the inference calls do (values within about 2e-3 of exact
 *   arithmetic).  Where two next actions' values lie closer than that, a* may be either of them; batch->next_action
 *   reports the one taken.
 *   dW   : fp32 [arn_param_count], overwritten with dLoss/dW in canonical order
 *   loss : fp32 [4], overwritten: {total, policy (or cross-entropy, or squared TD error), value mse, entropy}
 * loss_kind a2c/ppo need head PV; c51 needs head C51; dqn needs head Q or DUEL (ARN_ESHAPE otherwise). */
int arn_train_step_grads(const arn_config *cfg, const void *w_packed, const arn_batch *batch, int B,
                         int loss_kind, float *dW, float *loss,
                         void *workspace, size_t workspace_bytes, void *stream);

/* ---- Parameter update rules (appendix "Update Rule for Multi-Step Asynchronous Adam"; RMSProp as named in
 * appendix "Experiment Details" and in the appendix on update rules) ----
 * All arrays are device fp32 vectors of n entries, 16-byte aligned, updated in place; g is read only.
 * Arithmetic is fp32; the step-count dependent scalars are formed on the host in fp64.
 * Optional repack: if w_packed is not NULL, cfg must describe the network whose flat parameter vector theta
 * is (n == arn_param_count(cfg), else ARN_ESHAPE) and the packed copy is rewritten from the new theta on
 * the same stream, which makes a separate arn_weights_prepare call unnecessary.  With w_packed == NULL, cfg
 * is ignored and n is arbitrary (>= 1).
 * Errors: ARN_EINVAL for null/misaligned pointers, n == 0, t < 1, a decay outside [0,1), eps < 0. */

/* RMSProp without momentum, squared gradients accumulated directly:
 *   accu <- rho*accu + (1-rho)*g^2 ;  theta <- theta - lr*g / sqrt(accu + eps)      (eps inside the root)
 * accu starts at zero (the caller clears it).  eps = 0 with accu = 0 and g = 0 gives 0/0 = NaN, as the
 * formula does. */
int arn_rmsprop_update(size_t n, float *theta, const float *g, float *accu, float lr, float rho, float eps,
                       const arn_config *cfg, void *w_packed, void *stream);

/* Adam, first block of equations of the appendix, with t the step count AFTER the increment (1 on the first
 * call; the caller keeps it):
 *   a = r*sqrt(1-beta2^t)/(1-beta1^t);  m <- beta1*m + (1-beta1)*g;  v <- beta2*v + (1-beta2)*g^2;
 *   s = a*m/(sqrt(v) + eps);  theta <- theta - s.       m and v start at zero. */
int arn_adam_update(size_t n, float *theta, const float *g, float *m, float *v, int64_t t, float r, float beta1,
                    float beta2, float eps, const arn_config *cfg, void *w_packed, void *stream);

/* Local step of the multi-step asynchronous rule: the Adam step above on the learner's own theta, m, v plus
 * the second block of equations:  a_g <- beta1*a_g + g;  a_g2 <- beta2*a_g2 + g^2;  a_s <- a_s + s.
 * The accumulators start at zero. */
int arn_async_adam_local_step(size_t n, float *theta, const float *g, float *m, float *v, float *a_g, float *a_g2,
                              float *a_s, int64_t t, float r, float beta1, float beta2, float eps,
                              const arn_config *cfg, void *w_packed, void *stream);

/* Merge into the central values (third block of equations), n_local = local steps since the last merge:
 *   theta, theta_c <- theta_c - a_s;   m, m_c <- beta1^n_local*m_c + (1-beta1)*a_g;
 *   v, v_c <- beta2^n_local*v_c + (1-beta2)*a_g2;   a_g, a_g2, a_s <- 0.
 * The central arrays must be distinct from the local ones (ARN_EINVAL otherwise).  The call does not
 * serialise learners: two merges into the same central arrays that overlap in time race; order them on one
 * stream or with events.  The optional repack is of the learner's (new) theta. */
int arn_async_adam_merge(size_t n, float *theta_c, float *m_c, float *v_c, float *theta, float *m, float *v,
                         float *a_g, float *a_g2, float *a_s, int n_local, float beta1, float beta2,
                         const arn_config *cfg, void *w_packed, void *stream);

/* Optional instrumentation for benchmarks (not part of the paper's method).
 * While enabled, every kernel launch made by the calls above is bracketed by a
 * pair of HIP events on the caller's stream.  arn_profile_collect waits for the
 * recorded events (it DOES synchronise), writes up to `cap` records in launch
 * order -- names as HOST char[cap][32], durations in milliseconds as HOST
 * float[cap] -- frees the events and returns the number written.  Process-wide
 * state; not thread-safe. */
int arn_profile_enable(int on);
/* Records an event pair around no work on `stream` (name "null"): the instrumentation's own contribution to
 * every recorded duration, for the caller to subtract. */
int arn_profile_null(void *stream);
int arn_profile_collect(char *names, float *ms, int cap);

/* Human-readable name of a status code (static storage). */
const char *arn_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* ARN_H */
