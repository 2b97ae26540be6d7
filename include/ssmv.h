/*
 * ssmv.h - C ABI of the MI355X (gfx950) library for multi-step speculative
 * verification through a selective state-space (Mamba / Mamba-2) layer.
 *
 * The operations follow arXiv 2408.15237:
 *   Section 2.1, Eq. 1      h_t = A_t h_{t-1} + B_t x_t ,  y_t = C_t^T h_t
 *   Section 2.2             diagonal A, per-step sampling interval Delta_t; the
 *                           discrete parameters are rebuilt on the fly as
 *                           A_bar = exp(Delta_t * A), B_bar = Delta_t * B_t and
 *                           never stored
 *   Section 4.2, MultiStep  y_{j:k}, h_j, h_k <- MultiStep(h_i, ., i, j, k; A,B,C,Delta)
 *   Section 4.2, Alg. 2     Verify keeps ONE cached state and returns h_k when
 *                           every draft is accepted, else h_j; FirstConflict
 *   Section 4.3             recomputation of old steps, multi-step decoding of
 *                           the drafts and caching in ONE kernel; the conv part
 *                           of the block as a circular buffer
 *
 * Conventions
 *   - Every pointer inside ssmv_cache and every tensor argument is DEVICE memory
 *     owned by the CALLER (for instance torch tensors).  The library allocates
 *     and frees no device memory.  Pointers must be 16-byte aligned and stay
 *     valid until the stream has executed the call.  ssmv_dims and ssmv_cache are
 *     HOST structs, read during the call only.
 *   - All calls are asynchronous on `hip_stream` (a hipStream_t passed as void*,
 *     NULL = the default stream) except ssmv_check, which waits for the stream.
 *   - Arguments are validated on the host before any HIP call is made, so the
 *     error paths can be exercised without a GPU.  Every function returns an
 *     ssmv_status; ssmv_last_error() gives the text of the calling thread's
 *     last failure.
 *   - h_t is the state AFTER token t.  Per sequence, `pos` tokens are folded
 *     into the live state slot and `pend` more tokens are accepted but not yet
 *     folded (they sit in the current half of the pending-token window and are
 *     replayed by the next verify): the cache is advanced lazily.
 *   - One cache must not be used from two streams at once.  Per round the calls
 *     go conv1d_state_update -> ssm_verify_multistep -> ssm_commit_rollback.
 *     Verify changes neither the live slot nor any integer except last_k, so
 *     repeating it is legal and gives the same result.
 */
#ifndef SSMV_H
#define SSMV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SSMV_OK = 0,
    SSMV_EINVAL = -1,        /* null pointer, size or enum out of range                 */
    SSMV_EUNSUPPORTED = -2,  /* valid request that no compiled kernel covers            */
    SSMV_EALIGN = -3,        /* a device pointer is not 16-byte aligned                 */
    SSMV_ESEQUENCE = -4,     /* ssmv_check: the device saw a bad accepted[] / ordering  */
    SSMV_EHIP = -5           /* a HIP runtime call failed                               */
} ssmv_status;

enum { SSMV_F32 = 0, SSMV_BF16 = 1 };           /* io_dtype: storage type of tokens, y, conv ring, windows */
enum { SSMV_A_SCALAR = 0, SSMV_A_DIAG = 1 };    /* a_mode: A[H] (one decay per head) or A[H][N], headdim 1  */
enum { SSMV_ACT_NONE = 0, SSMV_ACT_SILU = 1 };  /* conv_act                                                */
/* snapshot_mode.  BOTH is Algorithm 2 as printed: verify stores h_j (when tokens were pending) and h_k, and a
 * fully accepted round makes h_k the live state.  HJ_ONLY never stores h_k: every accepted token, also those of
 * a fully accepted round, stays pending and is replayed by the next verify.  Same outputs and same logical
 * state; about a third fewer bytes per round for up to k more replay steps.
 * DEFER goes one step further along the lazily advanced single cached state of Section 4.2: h_k is never stored,
 * and h_j only when it has to be.  A verify recomputes up to SSMV_WINDOW
 * tokens from the cached state, so the live slot stays put and the accepted tokens collect behind it for as long as the
 * next round is sure to fit: a verify stores h_j (and its commit moves the live slot there) only if it meets
 * pend > SSMV_WINDOW - 2*kmax.  kmax <= SSMV_WINDOW/2; with kmax = SSMV_WINDOW/2 this is HJ_ONLY.  Same outputs and same
 * logical state; most rounds then only READ the state (kmax = 4, acceptance uniform in [0,4]: a store about every
 * fifth round).  The pending tokens of a sequence sit in a ring of SSMV_WINDOW entries (see ssmv_cache). */
enum { SSMV_SNAP_BOTH = 0, SSMV_SNAP_HJ_ONLY = 1, SSMV_SNAP_DEFER = 2 };
/* engine.  AUTO lets the library pick the kernel and with it the layout of the state slots: scalar-A mode with bf16
 * tokens, headdim a multiple of 64, dstate in {32, 64, 128} and kmax <= 8 (HJ_ONLY: pend can reach kmax, so 2*kmax <= 16)
 * runs the launch of Section 4.3 on the matrix cores and keeps each (sequence, head) block of a slot in 16x16 tiles;
 * everything else runs on the vector ALUs with row-major slots.  VECTOR forces the latter.  Same results to rounding. */
enum { SSMV_ENGINE_AUTO = 0, SSMV_ENGINE_VECTOR = 1 };

#define SSMV_KMAX_LIMIT 16      /* largest supported kmax                   */
#define SSMV_WINDOW 16          /* SSMV_SNAP_DEFER: tokens (pending + drafts) a verify can take, and entries of the window ring */
#define SSMV_CONV_WIDTH 4       /* the only supported conv width            */
#define SSMV_CACHE_NPTR 15      /* number of pointers in ssmv_cache         */

typedef struct {
    int32_t batch;          /* sequences                                                          */
    int32_t nheads;         /* H  (diag mode: the number of channels)                             */
    int32_t headdim;        /* P  (diag mode: must be 1)                                          */
    int32_t dstate;         /* N  in {16, 32, 64, 128, 256} (diag mode: <= 64)                     */
    int32_t ngroups;        /* G  B/C groups; H % G == 0; head hd uses group hd*G/H               */
    int32_t conv_width;     /* W  must be SSMV_CONV_WIDTH                                         */
    int32_t conv_channels;  /* Cx must equal H*P                                                  */
    int32_t kmax;           /* largest k ever passed, 1..SSMV_KMAX_LIMIT                          */
    int32_t ring_len;       /* R  power of two >= W-1+kmax                                        */
    int32_t io_dtype;       /* SSMV_F32 | SSMV_BF16                                               */
    int32_t a_mode;         /* SSMV_A_SCALAR | SSMV_A_DIAG                                        */
    int32_t conv_act;       /* SSMV_ACT_NONE | SSMV_ACT_SILU                                      */
    int32_t snapshot_mode;  /* SSMV_SNAP_BOTH | SSMV_SNAP_HJ_ONLY | SSMV_SNAP_DEFER               */
    int32_t engine;         /* SSMV_ENGINE_AUTO | SSMV_ENGINE_VECTOR                              */
} ssmv_dims;

/* The per-layer cache (Section 4.2: one cached state per sequence, advanced lazily;
 * Section 4.3 footnote: the conv inputs as a circular buffer). */
typedef struct {
    float   *state;        /* three slots of batch*H*P*N fp32, one block of P*N per (sequence, head); the order
                            * INSIDE a block is the library's (row-major or tiled, see `engine`): bring a state
                            * in with ssmv_cache_reset and take it out with ssmv_materialize               */
    void    *conv_ring;    /* [batch][R][Cx] io_dtype, channel fastest: raw conv inputs             */
    void    *win_xc[2];    /* [batch][kmax][Cx]   io_dtype: conv outputs of a round (ping-pong)     */
    void    *win_dt[2];    /* [batch][kmax][H]    io_dtype                                          */
    void    *win_B[2];     /* [batch][kmax][G][N] io_dtype                                          */
                           /* SSMV_SNAP_DEFER: win_*[0] is [batch][SSMV_WINDOW][..], a ring per sequence in which
                            * token q of the sequence (q = pos .. pos+pend-1 pending, then the round's) sits at
                            * entry q % SSMV_WINDOW; win_*[1] is not used (ssmv_cache_sizes asks for one granule) */
    int32_t *cur_slot;     /* [batch] in {0,1,2}: the live slot, holds the state at `pos`           */
    int32_t *pend;         /* [batch] in [0,kmax) (HJ_ONLY: [0,kmax]; DEFER: [0,SSMV_WINDOW-kmax]): accepted tokens not yet folded  */
    int64_t *pos;          /* [batch] tokens folded into state[cur_slot]                            */
    int32_t *conv_head;    /* [batch] ring index of the newest COMMITTED raw input                  */
    int32_t *last_k;       /* [batch] k of the verify that has not been committed yet, else 0       */
    int32_t *win_par;      /* [1] which half of win_* holds the pending tokens                      */
    int32_t *err_flag;     /* [1] sticky; set by the device on a bad accepted[] or a stray commit   */
} ssmv_cache;

/* Which kernel the verify launches of these dimensions run on, and with it the layout of the state slots (see
 * `engine`): 1 = matrix cores on tiled slots, 0 = vector ALUs on row-major slots; a negative ssmv_status for bad dims. */
int ssmv_engine_of(const ssmv_dims *dims);

/* Bytes the caller must allocate for each pointer of ssmv_cache, in declaration
 * order: state, conv_ring, win_xc[0], win_xc[1], win_dt[0], win_dt[1], win_B[0],
 * win_B[1], cur_slot, pend, pos, conv_head, last_k, win_par, err_flag.  Each size is
 * rounded up to a multiple of 256 bytes; the kernels may read (never write) up to
 * the end of the last granule. */
int ssmv_cache_sizes(const ssmv_dims *dims, size_t out_bytes[SSMV_CACHE_NPTR]);

/* Start a cache: slot 0 <- h0 ([batch][H][P][N] fp32 device, NULL = zeros), the
 * ring's first W-1 entries <- conv_init ([batch][W-1][Cx] io_dtype device, NULL
 * = zeros: an empty history), conv_head = W-2, every other integer 0
 * (Algorithm 2, Speculate: h_cache <- h_0, j <- 0). */
int ssmv_cache_reset(const ssmv_dims *dims, const ssmv_cache *cache, const float *h0,
                     const void *conv_init, void *hip_stream);

/* Conv roll (Section 4.3 footnote).  Appends the k raw inputs of this round to
 * the ring after conv_head[b] (older committed entries are kept, entries of a
 * rejected suffix are simply overwritten by the next round) and writes
 *   xc[b][t][c] = act(bias[c] + sum_{w<W} wgt[c][w] * raw_b[j_b+1+t-(W-1)+w][c]),
 * a causal depthwise cross-correlation over the committed inputs followed by
 * the new ones, accumulated in fp32 and rounded to io_dtype.
 *   x_raw [batch][k][Cx], wgt [Cx][W], bias [Cx] or NULL, xc_out [batch][k][Cx]:
 *   all io_dtype, device.  1 <= k <= kmax.  Integers of the cache are not changed. */
int conv1d_state_update(const ssmv_dims *dims, const ssmv_cache *cache, const void *x_raw,
                        const void *wgt, const void *bias, int32_t k, void *xc_out,
                        void *hip_stream);

/* MultiStep of Section 4.2 fused as Section 4.3 asks: in ONE kernel launch, per
 * sequence, (i) load the live state h_pos and replay the pend[b] pending tokens
 * from the window, (ii) if pend[b] > 0 (SSMV_SNAP_DEFER: > SSMV_WINDOW - 2*kmax) store that state h_j into slot
 * (cur+1)%3, (iii) run the k draft tokens
 *   h <- exp(dt_t*A) * h + (dt_t * x_t) (x) B_t ,   y_t = C_t . h + D * x_t
 * (Eq. 1; fp32 state and arithmetic), (iv) store h_k into slot (cur+2)%3 (SSMV_SNAP_BOTH
 * only) and this round's (xc, dt, B) into the other half of the window (DEFER: behind the pending ones in the ring).  Intermediate
 * states and the discrete parameters live in registers/LDS only.
 *   xc [batch][k][H*P], dt [batch][k][H], Bm, Cm [batch][k][G][N]: io_dtype, device;
 *   dt is the final positive step size; A [H] or [H][N] (negative reals) and D [H]:
 *   fp32, device; y_out [batch][k][H*P] io_dtype.  1 <= k <= kmax.
 * Sets last_k[b] = k; changes no other integer and not the live slot. */
int ssm_verify_multistep(const ssmv_dims *dims, const ssmv_cache *cache, const void *xc,
                         const void *dt, const void *Bm, const void *Cm, const float *A,
                         const float *D, int32_t k, void *y_out, void *hip_stream);

/* conv1d_state_update and ssm_verify_multistep in ONE launch (Section 4.3: the
 * paper fuses recomputation, multi-step decoding and caching; the conv roll over
 * the circular buffer is folded into the same kernel's token staging here).
 * Takes the raw conv inputs instead of xc: x_raw [batch][k][Cx], wgt [Cx][W],
 * bias [Cx] or NULL (io_dtype, device).  Appends x_raw to the ring, computes
 * xc exactly as conv1d_state_update does (same fp32 order, same rounding),
 * stashes it in the window, and runs the verification on it.  xc itself is not
 * returned.  Everything else as for ssm_verify_multistep. */
int ssm_conv_verify_multistep(const ssmv_dims *dims, const ssmv_cache *cache, const void *x_raw,
                              const void *wgt, const void *bias, const void *dt, const void *Bm,
                              const void *Cm, const float *A, const float *D, int32_t k,
                              void *y_out, void *hip_stream);

/* The general form of the two calls above, with the optional pieces that make the launch a whole
 * Mamba block's recurrence and that let a round be fed by several calls:
 *   - dt <- softplus(dt + dt_bias) ahead of the discretisation (Section 2.2 takes the positive step
 *     size as given; a Mamba block obtains it this way).  dt_bias [H] (diag mode: per channel) fp32 device
 *     or NULL (= 0); dt_softplus 0/1.  The window keeps the raw dt and replay transforms it again, so
 *     both must be the same on every call on one cache, ssmv_materialize_block included;
 *   - y <- y * z * sigmoid(z), the block's SiLU gate, in fp32 ahead of the rounding of y.
 *     z [batch][k][H*P] io_dtype device, or NULL for no gate;
 *   - tok0 > 0: the draft side (Section 4.3: a draft model that is itself an SSM produces one token
 *     per call, and its first call of a round recomputes the tokens accepted last round).  The first
 *     call of a round has tok0 = 0 and is a verify as above; a later call, with tok0 = the number
 *     of tokens the round has been fed so far, continues from the state in the h_k slot, updates that
 *     slot in place, replays nothing, appends its k tokens to the round's window and conv ring, and sets
 *     last_k[b] = tok0 + k.  After the calls the window, the ring and the integers hold exactly what one
 *     call with all tok0+k tokens would have left, the slots and the outputs the same up to fp32 rounding
 *     (the rounding order inside a launch depends on how many tokens it holds), so ssm_commit_rollback
 *     applies unchanged.
 *     tok0 + k <= kmax; SSMV_SNAP_BOTH only (SSMV_EUNSUPPORTED otherwise); a later call is NOT idempotent.
 *   - replay_round = 1 (matrix-core engine only, SSMV_EUNSUPPORTED otherwise): the other way to feed a round by
 *     several calls, the one Section 4.3 describes for the draft model - recompute from the cache instead of
 *     carrying the state through memory.  EVERY call of the round starts from the live slot, replays the pending
 *     tokens and the tok0 tokens the round has been fed so far (their conv outputs, dt and B sit in the round's
 *     half of the window), then takes its k tokens; it stores no state unless last_call = 1, which stores h_j and
 *     h_k as one call with all tok0 + k tokens would.  A call then reads the state once and writes it only at the
 *     end of the round (the default above reads and writes it on every call).  Calls are idempotent.  All calls
 *     of a round must agree on replay_round, and the round must end with a last_call = 1 before its commit.
 *     Works with SSMV_SNAP_HJ_ONLY and SSMV_SNAP_DEFER too.
 *   - k_seq (device int32 [batch], or NULL): ragged draft counts.  Sequence b takes only the first
 *     kb = clamp(k_seq[b], 1, k) of the k tokens given (at least one: last_k = 0 means "no verify"
 *     to the commit; a sequence with nothing to verify passes one token and accepts none) (the arrays keep the stride k): its outputs
 *     y[b][t >= kb] are written as zeros, its h_k slot holds the state after kb tokens, last_k[b] =
 *     tok0 + kb, and ssm_commit_rollback then clamps accepted[b] to that.  Work for the tokens
 *     not taken is skipped.  Not together with tok0 > 0 (SSMV_EUNSUPPORTED).
 * Exactly one of x_raw (conv fused; needs conv_wgt) and xc is non-NULL.  Other arguments as above. */
typedef struct ssmv_step_args {
    const void *x_raw;      /* [batch][k][Cx] io_dtype, or NULL */
    const void *xc;         /* [batch][k][H*P] io_dtype, or NULL */
    const void *conv_wgt;   /* [Cx][W] io_dtype (with x_raw) */
    const void *conv_bias;  /* [Cx] io_dtype or NULL */
    const void *dt;         /* [batch][k][H] io_dtype */
    const float *dt_bias;   /* [H] fp32 or NULL */
    const void *Bm;         /* [batch][k][G][N] io_dtype */
    const void *Cm;         /* [batch][k][G][N] io_dtype */
    const void *z;          /* [batch][k][H*P] io_dtype or NULL */
    const float *A;         /* [H] or [H][N] fp32 */
    const float *D;         /* [H] fp32 */
    const int32_t *k_seq;   /* [batch] int32 or NULL */
    void *y_out;            /* [batch][k][H*P] io_dtype */
    int32_t k;
    int32_t tok0;
    int32_t dt_softplus;
    int32_t replay_round;   /* 0 | 1 */
    int32_t last_call;      /* with replay_round = 1: 1 on the round's last call */
} ssmv_step_args;
int ssm_block_multistep(const ssmv_dims *dims, const ssmv_cache *cache, const ssmv_step_args *args,
                        void *hip_stream);

/* Prefill: all L prompt tokens of every sequence through the layer (Section 2.1 Eq. 1 with the
 * discretisation of Section 2.2, evaluated chunk by chunk on the matrix cores), so that decoding can
 * start from the cache.  Computes the conv roll and every y_t, advances the LIVE slot in place by
 * the L tokens, leaves the newest conv_width-1 raw inputs in the ring, and (in a second, tiny launch)
 * sets pos[b] += L and conv_head[b] += L.  The cache must hold no pending tokens and no uncommitted
 * verify (pend[b] = last_k[b] = 0), else err_flag is set.  Scalar a_mode, headdim and dstate in
 * {32, 64, 128} (SSMV_EUNSUPPORTED otherwise); L >= 1, the same for all sequences.
 * Arithmetic: fp32 tensors multiply in fp32; bf16 tensors multiply on the bf16 matrix cores with
 * fp32 accumulation, B, C and the conv output entering exactly.  The fp32 operand of the product that
 * updates the state enters as a bf16 head plus a bf16 tail, which keeps 2^-17 of it: the state stays
 * within about 1e-4 (relative) of the exact scan.  The fp32 operands of the products that end in outputs
 * only enter as their bf16 head (2^-9 per term, the size of the outputs' own bf16 rounding): an output is
 * within about 1e-2 of the largest output of its tensor.
 * dt is the positive step (after softplus, if that is requested); an input that is not finite
 * anywhere in a chunk of 32 tokens can spread over that chunk's outputs.
 *   x_raw, y_out [batch][L][H*P]; dt [batch][L][H]; Bm, Cm [batch][L][G][N]: io_dtype, device;
 *   wgt [Cx][W], bias [Cx] or NULL; A, D [H] fp32. */
int ssm_prefill_chunked(const ssmv_dims *dims, const ssmv_cache *cache, const void *x_raw,
                        const void *wgt, const void *bias, const void *dt, const void *Bm,
                        const void *Cm, const float *A, const float *D, int32_t L, void *y_out,
                        void *hip_stream);

/* The general form of the prefill: the block pieces of ssm_block_multistep (dt <- softplus(dt +
 * dt_bias); y <- y * z * sigmoid(z) in fp32 ahead of the rounding of y) and prompts of different
 * lengths.  seq_len (device int32 [batch], or NULL = all L): sequence b feeds its first
 * clamp(seq_len[b], 0, L) tokens; the arrays keep the token stride L, outputs behind a sequence's
 * length are not written, its pos and conv_head advance by its own length, and a sequence of
 * length 0 is left untouched. */
typedef struct ssmv_prefill_args {
    const void *x_raw;      /* [batch][L][Cx] io_dtype */
    const void *conv_wgt;   /* [Cx][W] io_dtype */
    const void *conv_bias;  /* [Cx] io_dtype or NULL */
    const void *dt;         /* [batch][L][H] io_dtype */
    const float *dt_bias;   /* [H] fp32 or NULL */
    const void *Bm;         /* [batch][L][G][N] io_dtype */
    const void *Cm;         /* [batch][L][G][N] io_dtype */
    const void *z;          /* [batch][L][H*P] io_dtype or NULL */
    const float *A;         /* [H] fp32 */
    const float *D;         /* [H] fp32 */
    const int32_t *seq_len; /* [batch] int32 or NULL */
    void *y_out;            /* [batch][L][H*P] io_dtype */
    int32_t L;
    int32_t dt_softplus;
} ssmv_prefill_args;
int ssm_prefill_block(const ssmv_dims *dims, const ssmv_cache *cache, const ssmv_prefill_args *args,
                      void *hip_stream);

/* Algorithm 2, "return h_k if k' = k else h_j", as integer bookkeeping.  Per
 * sequence with a = accepted[b] (device int32 [batch]; values outside
 * [0,last_k] are clamped and set err_flag):
 *   a == last_k : cur <- (cur+2)%3, pos <- pos+pend+a, pend <- 0
 *   pend > 0    : cur <- (cur+1)%3, pos <- pos+pend,   pend <- a
 *   otherwise   :                                      pend <- a
 *   always      : conv_head <- (conv_head+a) & (R-1), last_k <- 0
 * and win_par flips once.  A commit with no verify pending changes nothing and
 * sets err_flag.  With SSMV_SNAP_HJ_ONLY the first case does not exist: pend > 0
 * moves to h_j as above, and pend <- a in every case.  With SSMV_SNAP_DEFER:
 *   pend > SSMV_WINDOW - 2*kmax : cur <- (cur+1)%3, pos <- pos+pend, pend <- a      (the verify stored h_j)
 *   otherwise                   :                                    pend <- pend+a */
int ssm_commit_rollback(const ssmv_dims *dims, const ssmv_cache *cache, const int32_t *accepted,
                        void *hip_stream);

/* The same commit for n_caches caches that share dims and the accepted lengths
 * (the SSM layers of one model: acceptance is decided per sequence, once, after
 * the last layer), in one launch per 32 caches.  `caches` is a HOST array. */
int ssm_commit_rollback_multi(const ssmv_dims *dims, const ssmv_cache *caches, int32_t n_caches,
                              const int32_t *accepted, void *hip_stream);

/* State at pos+pend (live slot with the pending tokens folded in), written to
 * h_out [batch][H][P][N] fp32 device; the cache is not changed.  For tests and
 * for handing the state to another engine. */
int ssmv_materialize(const ssmv_dims *dims, const ssmv_cache *cache, const float *A, float *h_out,
                     void *hip_stream);
/* The same for a cache that is driven with a dt transform (see ssm_block_multistep). */
int ssmv_materialize_block(const ssmv_dims *dims, const ssmv_cache *cache, const float *A,
                           const float *dt_bias, int32_t dt_softplus, float *h_out, void *hip_stream);

/* The norm that follows the recurrence in a Mamba-2 block (outside the verify launch: it reduces over
 * all heads of a token, i.e. across that launch's workgroups): per token row and per group of
 * group_size adjacent channels,  g = y * z * sigmoid(z)  (g = y when z is NULL, e.g. because the
 * verify launch already applied the gate),  out = g * rsqrt(mean(g^2) + eps) * weight,  fp32
 * arithmetic, out rounded to io_dtype.  y, z, out [rows][channels] io_dtype device (out may be y);
 * weight [channels] fp32 device.  group_size a multiple of 8 (bf16) or 4 (fp32), at most 8192 / 4096. */
int ssmv_gated_rmsnorm(const void *y, const void *z, const float *weight, int32_t rows, int32_t channels,
                       int32_t group_size, float eps, int32_t io_dtype, void *out, void *hip_stream);

/* FirstConflict of Algorithm 2: accepted[b] = length of the longest prefix on
 * which draft[b][.] and target[b][.] agree.  draft, target [batch][k] and
 * accepted [batch]: int32, device. */
int ssmv_first_conflict(const int32_t *draft, const int32_t *target, int32_t batch, int32_t k,
                        int32_t *accepted, void *hip_stream);

/* Waits for the stream and returns SSMV_ESEQUENCE if err_flag is set, else SSMV_OK. */
int ssmv_check(const ssmv_cache *cache, void *hip_stream);

/* Launch shape of the verify kernel.  rows_per_lane in {0 = choose from the
 * problem size, 1, 2, 4, 8}; waves_per_group in {0 = choose, 1, 2, 4}.  Process-wide;
 * for tuning and for tests that want to cover every shape. */
int ssmv_set_tuning(int32_t rows_per_lane, int32_t waves_per_group);

/* Plain device copy kernel used to calibrate bandwidth counters and the
 * achievable HBM ceiling: reads n_bytes from src, writes them to dst0 and, if
 * dst1 is not NULL, to dst1 as well (the verify kernel's read-S / write-2S
 * pattern).  n_bytes must be a multiple of 16. */
int ssmv_copy_probe(const void *src, void *dst0, void *dst1, size_t n_bytes, void *hip_stream);

/* Bandwidth probe for the ceiling the measurements are held against: one launch streams n_bytes in the given direction,
 * non-temporal like the state traffic of the verify kernel.  READ reads src (dst0 must be a valid pointer, it is not
 * written); WRITE writes dst0; R1W1 copies src to dst0; R1W2 to dst0 and dst1; EMPTY launches the same grid and does
 * nothing (the cost of a launch).  A workgroup takes contiguous pieces of piece_kib in {4, 8, 32} KiB; grid = 0 launches
 * one workgroup per piece, grid > 0 that many workgroups looping over the pieces.  n_bytes: a multiple of the piece. */
enum { SSMV_PROBE_READ = 0, SSMV_PROBE_WRITE = 1, SSMV_PROBE_R1W1 = 2, SSMV_PROBE_R1W2 = 3, SSMV_PROBE_EMPTY = 4 };
int ssmv_stream_probe(int32_t mode, const void *src, void *dst0, void *dst1, size_t n_bytes, int32_t piece_kib, int32_t grid,
                      void *hip_stream);

const char *ssmv_last_error(void);
const char *ssmv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SSMV_H */
