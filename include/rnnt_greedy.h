/*
 * rnnt_greedy.h -- C ABI of the MI355X (gfx950) engine for exact batched
 * RNN-T / TDT greedy decoding.
 *
 * The library runs the whole data-dependent decoding loop of the paper
 * "Speed of Light Exact Greedy Decoding for RNN-T Speech Recognition Models on
 * GPU" on the device: one launch of the encoder-side joint projection and one
 * launch of a persistent decode kernel per call, no host round trip per step
 * (the paper's Section "Algorithm Implementation" explains why the per-step
 * host contact is what makes the baseline slow).
 *
 * Conventions
 *   - All pointers named in rnnt_model_desc and all tensor arguments of the
 *     decode calls are DEVICE pointers unless marked HOST.  fp32, row-major.
 *   - Linear and LSTM weights are [out, in]; LSTM gate order along `out` is
 *     input, forget, cell, output (i, f, g, o); two bias vectors per layer.
 *   - The caller owns every buffer it passes and keeps it alive until the work
 *     queued on `stream` has finished.  The engine owns its packed copy of the
 *     weights and its workspace; decode calls allocate nothing.
 *   - Decode calls only enqueue work on `stream` and return; they never wait
 *     for the device and never read device memory from the host.
 *   - One engine serves one call at a time (shared workspace): calls on the
 *     same engine must be ordered by the caller (same stream or events).  A
 *     decode launch occupies every compute unit, so calls of different engines
 *     gain nothing from running on different streams; order them too.
 *   - Return value: RNNT_OK (0) or a negative RNNT_ERR_* code, detected on the
 *     host before anything is queued.  Conditions only the device can see are
 *     reported through rnnt_engine_status().
 */
#ifndef RNNT_GREEDY_H
#define RNNT_GREEDY_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rnnt_engine rnnt_engine;
/* A hipStream_t, passed as an opaque pointer so this header needs no HIP. */
typedef void *rnnt_stream_t;

enum {
    RNNT_OK = 0,
    RNNT_ERR_NULL = -1,        /* a required pointer is NULL                   */
    RNNT_ERR_SHAPE = -2,       /* a dimension or count is out of range         */
    RNNT_ERR_VARIANT = -3,     /* the decoder does not run this kind of model  */
    RNNT_ERR_HIP = -4,         /* a HIP runtime call failed                    */
    RNNT_ERR_UNSUPPORTED = -5, /* the device or the model does not fit         */
    RNNT_ERR_SCRATCH = -6      /* rnnt_label_looping_decode_noalloc: the call  */
                               /* needs more than the static scratch array     */
};

/* Bits of the device status word (rnnt_engine_status). */
enum {
    RNNT_DEV_LEN_CLAMPED = 1,   /* some enc_len[b] was outside [0, T]           */
    RNNT_DEV_OVERFLOW = 2,      /* more tokens than `cap`; the excess is dropped */
    RNNT_DEV_ABORTED = 4        /* a bounded wait expired: outputs are invalid   */
};

/* Flags of rnnt_engine_create. */
enum {
    RNNT_FLAG_DEFAULT = 0
};

/*
 * The decoder's weights (prediction network = embedding + L stacked LSTM
 * layers; joint = W_out relu(W_enc f + b_enc + W_pred g + b_pred) + b_out,
 * the structure behind the paper's prediction() and joint() in Algorithm 1).
 * HOST struct holding DEVICE pointers; everything is copied and repacked by
 * rnnt_engine_create, so the struct and the weights may be freed afterwards.
 */
typedef struct rnnt_model_desc {
    int32_t F;       /* encoder output features                                */
    int32_t E;       /* embedding width                                        */
    int32_t H;       /* LSTM hidden width                                      */
    int32_t L;       /* LSTM layers (1..4)                                     */
    int32_t J;       /* joint hidden width                                     */
    int32_t V1;      /* vocabulary size including blank                        */
    int32_t blank;   /* blank index in [0, V1); also the start-of-sequence     */
                     /* label fed to the prediction network first              */
    int32_t D;       /* number of durations: 0 = RNN-T, >0 = TDT (at most 8)   */
    const int32_t *durations;      /* HOST, [D], e.g. {0,1,2,3,4}              */
    const float *emb;              /* [V1, E]                                  */
    const float *const *w_ih;      /* HOST array of L device pointers [4H,in_l] */
    const float *const *w_hh;      /* HOST array of L device pointers [4H, H]  */
    const float *const *b_ih;      /* HOST array of L device pointers [4H]     */
    const float *const *b_hh;      /* HOST array of L device pointers [4H]     */
    const float *w_enc, *b_enc;    /* [J, F], [J]                              */
    const float *w_pred, *b_pred;  /* [J, H], [J]                              */
    const float *w_out, *b_out;    /* [V1 + D, J], [V1 + D]; token logits      */
                                   /* first, then the D duration logits        */
} rnnt_model_desc;

/* Work counters of the last decode call (rnnt_engine_stats). */
typedef struct rnnt_stats {
    int64_t pred_steps;   /* batched prediction-network steps, summed over teams */
    int64_t joint_steps;  /* batched joint steps (chunks), summed over the first */
                          /* joint group of every team                           */
    int64_t max_pred_steps;   /* the same, for the team that did the most        */
    int64_t max_joint_steps;
    int64_t joint_samples;    /* (utterance, frame) pairs the joint evaluated    */
    int64_t barrier_polls;    /* polls spent in team barriers                    */
    int32_t n_teams;          /* work-group teams used by the call               */
    int32_t team_size;        /* work-groups per team                            */
    int32_t lookahead;        /* frames examined per utterance per joint step    */
    int32_t xcd_mismatch;     /* work-groups not on the XCD their weights are on */
    int32_t joint_groups;     /* groups per team that search for labels on their */
                              /* own (1 = the whole team together)               */
    int32_t search_steps;     /* joint steps a label search may take before the  */
                              /* next prediction step (0 = no limit)             */
    float projection_ms;      /* device time of the encoder-projection kernel    */
    float decode_ms;          /* device time of the persistent decode kernel,    */
                              /* both from HIP events recorded on the call's     */
                              /* stream around each launch                       */
} rnnt_stats;

/*
 * Engine flags.  RNNT_FLAG_BF16_WEIGHTS: keep the weights that are streamed at
 * every step (W_hh of every layer, W_ih of the layers above the first, W_pred,
 * W_out) as bf16 in the engine's packed copy, half the bytes per step.  The
 * storage is lossless or refused: every one of those weights must already be
 * a bf16 value (low 16 bits of the float zero), otherwise create returns
 * RNNT_ERR_SHAPE; the arithmetic stays fp32 (a stored weight is widened before
 * use), so the results are those of the fp32 engine on the same model up to
 * summation order.  The embedding, W_ih of the first layer, W_enc and all
 * biases may hold any fp32 values.  The paper's experiments run bf16 models
 * (section on the experimental set-up); this is the storage half of that.
 */
#define RNNT_FLAG_BF16_WEIGHTS 1

/*
 * rnnt_engine_create flag: the same matrices are kept as 8-bit floats in the
 * OCP e4m3 format (1 sign, 4 exponent, 3 mantissa bits; largest value 448, no
 * scale factors), a quarter of the fp32 bytes per step.  Lossless or refused
 * like the bf16 flag: every streamed weight must be an e4m3 value or create
 * returns RNNT_ERR_SHAPE; the arithmetic stays fp32.  Weight-only 8-bit storage
 * is the direction the paper's conclusion names for the next speed-up (there
 * for the encoder's products).  The two storage flags exclude each other
 * (RNNT_ERR_SHAPE).
 */
#define RNNT_FLAG_FP8_WEIGHTS 2

/*
 * rnnt_engine_create flag: bfloat16 mode (the precision the paper's experiments
 * run in, section on the experimental set-up).  Any fp32 model is accepted.
 * The weight matrices of all dense products -- embedding table, W_ih and W_hh of
 * every layer, W_enc, W_pred, W_out -- are rounded to bfloat16 (ties to even)
 * when the engine is created and the streamed ones are stored as bf16; every
 * vector that enters a product (encoder frames, hidden vectors, the joint's
 * hidden vector) is rounded to bfloat16 at that point.  Products are then exact
 * in fp32; sums, biases, activations, logits and the argmax stay fp32.  The
 * results are those of the fp32 engine on another arithmetic: token sequences
 * may differ from the fp32 decode of the same model, and are exact against a
 * reference that rounds at the same places (up to summation order).  Excludes
 * RNNT_FLAG_BF16_WEIGHTS (RNNT_ERR_SHAPE).  Together with RNNT_FLAG_FP8_WEIGHTS
 * it is the weight-only 8-bit form of the mode (the quantised products of the
 * paper's conclusion): the streamed weights are kept as e4m3 codes with one
 * power-of-two scale per weight row (per output of the product).  The engine
 * finds the scale itself -- 2^k with the smallest k for which the row's largest
 * magnitude times 2^-k is at most 448 -- and every weight of the row times 2^-k
 * must then be an e4m3 value, else RNNT_ERR_SHAPE (lossless or refused, per
 * row; rnnt_quantize_rows_e4m3 below maps any matrix to the nearest such one).
 * The codes are widened to bf16 and multiplied by the row's power of two in one
 * instruction on their way to the bf16 matrix instructions, without rounding;
 * the arithmetic is that of the bfloat16 mode on that model.
 */
#define RNNT_FLAG_BF16_ARITHMETIC 8

/*
 * Weight-only 8-bit quantisation of a matrix for the flags above (a host-side
 * helper; nothing runs on the device).  w and out are HOST arrays of
 * rows * cols floats, row-major, one row per output of the product; they may
 * be the same array.  For each row: k is the smallest integer with
 * max|row| * 2^-k <= 448 (0 for a row of zeros; kept within +-100), and every
 * weight becomes 2^k times the e4m3 value nearest to weight * 2^-k (ties to the even code).
 * scales_out, if not NULL, receives the rows' 2^k.  An engine created with
 * RNNT_FLAG_BF16_ARITHMETIC | RNNT_FLAG_FP8_WEIGHTS accepts the result for
 * any of its streamed matrices.  Weights that are not finite are
 * RNNT_ERR_SHAPE; NULL arrays RNNT_ERR_NULL.
 */
int rnnt_quantize_rows_e4m3(const float *w, int64_t rows, int64_t cols, float *out, float *scales_out);

/*
 * rnnt_engine_create flag, only together with RNNT_FLAG_BF16_ARITHMETIC (alone,
 * or with another format flag, RNNT_ERR_SHAPE): the weight-only 4-bit form of
 * the bfloat16 mode.  The streamed weights are kept as codes of the OCP e2m1
 * format (1 sign, 2 exponent, 1 mantissa bit: magnitudes 0, 0.5, 1, 1.5, 2, 3,
 * 4, 6) with one power-of-two scale per block of RNNT_FP4_BLOCK consecutive
 * weights of a row (the last block of a row may be shorter).  The engine finds
 * the scales itself -- 2^k with the smallest k for which the block's largest
 * magnitude times 2^-k is at most 6 -- and every weight of the block times 2^-k
 * must be an e2m1 value, else RNNT_ERR_SHAPE; rnnt_quantize_blocks_e2m1 maps
 * any matrix to the nearest such one.  Codes are widened to bf16 and scaled in
 * one instruction, without rounding; the arithmetic is the bfloat16 mode's on
 * that model.
 */
#define RNNT_FLAG_FP4_WEIGHTS 32
#define RNNT_FP4_BLOCK 128

/*
 * Weight-only 4-bit quantisation of a matrix for RNNT_FLAG_FP4_WEIGHTS (host
 * side, as rnnt_quantize_rows_e4m3): every block of RNNT_FP4_BLOCK consecutive
 * weights of a row becomes 2^k times the e2m1 values nearest to the weights
 * times 2^-k (ties to the even code), k the smallest integer with
 * max|block| * 2^-k <= 6 (0 for zeros; kept within +-100).  scales_out, if not
 * NULL, receives rows * ceil(cols / RNNT_FP4_BLOCK) values 2^k, row-major.
 */
int rnnt_quantize_blocks_e2m1(const float *w, int64_t rows, int64_t cols, float *out, float *scales_out);

/*
 * rnnt_engine_create flag: launch the decode kernel with an ordinary launch
 * instead of a cooperative one.  The kernel's teams synchronise among
 * themselves, which needs all work-groups resident at once; the cooperative
 * launch guarantees that, an ordinary launch of one work-group per compute
 * unit has it on a device that runs nothing else (every wait in the kernel is
 * bounded, so a call that does not get it ends with RNNT_DEV_ABORTED instead
 * of hanging).  For profiling runs: a process that has run a cooperative
 * launch under rocprofv3's kernel trace has been seen to crash in its exit
 * handlers.  May be combined with a storage flag.
 */
#define RNNT_FLAG_PLAIN_LAUNCH 4

/*
 * RNNT_FLAG_MULTI_BLANK: the model is a multi-blank transducer (the paper's
 * related-work section names these models beside TDT: "big blank" symbols let
 * the decoder skip encoder frames).  The D extra output columns of the
 * descriptor are then not durations but big-blank symbols, and durations[i]
 * (>= 1, else RNNT_ERR_SHAPE) is the number of frames big blank i skips.  All
 * V1 + D outputs form one distribution with one argmax (lowest index on
 * ties); a blank moves on by one frame and a big blank by its span, neither is
 * emitted or fed to the prediction network, both reset the count of labels on
 * the frame; a label is handled as in an RNN-T.  The log-probability output,
 * when set, is taken over all V1 + D outputs.  Such an engine is decoded with
 * rnnt_label_looping_decode (or its _noalloc form); rnnt_greedy_decode --
 * Algorithm 1 keeps one frame index for the whole batch -- and
 * tdt_label_looping_decode return RNNT_ERR_VARIANT.  May be combined with the
 * other flags.
 */
#define RNNT_FLAG_MULTI_BLANK 16

/*
 * Create an engine for up to max_B utterances of up to max_T frames.
 * Copies and repacks the weights on the current device, allocates the
 * workspace (projected frames [max_B, max_T, J], state, exchange buffers).
 * flags: 0 or one of RNNT_FLAG_BF16_WEIGHTS / RNNT_FLAG_FP8_WEIGHTS /
 * RNNT_FLAG_BF16_ARITHMETIC (or the last with RNNT_FLAG_FP8_WEIGHTS or
 * RNNT_FLAG_FP4_WEIGHTS), optionally with
 * RNNT_FLAG_PLAIN_LAUNCH and RNNT_FLAG_MULTI_BLANK; other bits are
 * RNNT_ERR_SHAPE.
 * Limits of this implementation, checked here before anything is allocated
 * (RNNT_ERR_UNSUPPORTED): F must be a multiple of 16 (K tile of the projection
 * GEMM); H and J multiples of 4 (rows are read 16 bytes at a time); V1 + D at
 * most 65 535 (the argmax exchange carries a 16-bit column index);
 * max_B * max_T below 2^31 (frame numbers are 32-bit); the device must
 * support cooperative launches.  1 <= L <= 4, D <= 8, blank in
 * [0, V1) and positive sizes are RNNT_ERR_SHAPE.
 * The two bias vectors of an LSTM layer are added once on the host while the
 * weights are repacked (b_ih + b_hh in fp32).
 * max_B itself has no limit but memory (the projected frames take
 * max_B * max_T * J floats): a call with more than 128 utterances is decoded
 * by consecutive launches of up to 128 utterances each, in the caller's order,
 * after one projection of the whole batch (on MI355X that is faster than
 * larger launches); status word and statistics cover the whole call, and
 * completion flags are raised launch by launch.  The state of a team of
 * work-groups has to fit the compute units' local memory: a model whose
 * state for 128 utterances fits in no team layout is decoded in launches of
 * the largest size that does fit (64, 16, ...), and one for which not even
 * the layout for two utterances fits returns RNNT_ERR_UNSUPPORTED.  The argmax
 * candidates of a joint step sit there too, one per sample and group of four
 * output columns of a rank: vocabularies of a few thousand labels fit for any
 * batch, tens of thousands only for engines of a few utterances.  When the
 * preferred team layout does not fit, the engine tries the others that divide
 * the device (fewer joint groups, then more teams, then fewer) before it
 * refuses.
 * Device memory of an engine: the projected frames (max_B * max_T * J floats)
 * and, per team layout (up to eleven, see rnnt_engine_configure), a packed
 * copy of the streamed weights and a few megabytes of workspace: about
 * 0.4 GB besides the projected frames for the Parakeet shape in fp32.
 * Synchronous.  *out is set only on success.
 */
int rnnt_engine_create(const rnnt_model_desc *desc, int32_t max_B, int32_t max_T,
                       int32_t flags, rnnt_engine **out);

/* Free the engine's device memory.  Synchronises the device first. */
int rnnt_engine_destroy(rnnt_engine *eng);

/*
 * Frame-looping greedy decoding: Algorithm 1 of the paper.  An outer loop over
 * frames shared by the utterances of a team, an inner loop of at most
 * max_symbols steps that ends when every utterance has produced a blank.
 *
 *   enc_out     [B, T, F]   encoder output, 16-byte aligned (the projection
 *                           kernel loads four floats at a time; any other
 *                           address is RNNT_ERR_SHAPE); frames t >= enc_len[b]
 *                           are padding and may hold anything, NaN included
 *   enc_len     [B]         valid frames per utterance; values outside [0, T]
 *                           are clamped on the device (RNNT_DEV_LEN_CLAMPED)
 *   tokens_out  [B, cap]    emitted labels in order; entries at and beyond
 *                           tok_len_out[b] are set to -1
 *   tok_len_out [B]         number of labels emitted (counts labels dropped
 *                           for lack of room too; cap >= T * max_symbols
 *                           always suffices)
 *   frames_out  [B, cap]    or NULL: frame index of each label
 *   logit_out   [B, cap]    or NULL: the winning (maximum) token logit
 * Errors: RNNT_ERR_NULL, RNNT_ERR_SHAPE (B, T outside the engine's limits,
 * max_symbols < 1, cap < 1), RNNT_ERR_VARIANT on a TDT engine.
 */
int rnnt_greedy_decode(rnnt_engine *eng, const float *enc_out, const int32_t *enc_len,
                       int32_t B, int32_t T, int32_t max_symbols,
                       int32_t *tokens_out, int32_t *tok_len_out, int32_t cap,
                       int32_t *frames_out, float *logit_out, rnnt_stream_t stream);

/*
 * Label-looping greedy decoding (the schedule described at the end of the
 * paper's Related Work section: every utterance advances its own frame index,
 * the outer loop runs once per label, the inner loop skips blanks).  Same
 * arguments and the same outputs, token for token, as rnnt_greedy_decode.
 */
int rnnt_label_looping_decode(rnnt_engine *eng, const float *enc_out, const int32_t *enc_len,
                              int32_t B, int32_t T, int32_t max_symbols,
                              int32_t *tokens_out, int32_t *tok_len_out, int32_t cap,
                              int32_t *frames_out, float *logit_out, rnnt_stream_t stream);

/*
 * rnnt_label_looping_decode for callers that cannot allocate device memory or
 * have it allocated on their behalf: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * outputs, same errors.  The call's scratch -- the projected frames
 * [B, T, J] and what the teams exchange -- does not come from the engine's
 * workspace but from one array of RNNT_NOALLOC_SCRATCH_BYTES bytes that the
 * library holds as a static device object on every device it runs on, until
 * the process ends.  The entry point calls no hipMalloc, hipFree or other
 * allocating routine; the engine (its packed weights) is created beforehand.
 * A call that needs more (roughly B * T * J * 4 bytes plus 9 MiB at the
 * Parakeet shape), or one of more than 128 utterances (it would take more than
 * one launch), returns RNNT_ERR_SCRATCH and queues nothing.
 * All calls on one device share the array, which keeps the last call's
 * contents (the call clears what must start at zero): calls through this entry
 * point that overlap on one device race, whatever engines and streams they use;
 * order them.  rnnt_engine_status / rnnt_engine_stats report on such a call
 * until the next call on the engine.
 */
#define RNNT_NOALLOC_SCRATCH_BYTES (32u << 20)
int rnnt_label_looping_decode_noalloc(rnnt_engine *eng, const float *enc_out,
                                      const int32_t *enc_len, int32_t B, int32_t T,
                                      int32_t max_symbols, int32_t *tokens_out,
                                      int32_t *tok_len_out, int32_t cap, int32_t *frames_out,
                                      float *logit_out, rnnt_stream_t stream);

/*
 * Label-looping decoding of a token-and-duration transducer (the TDT rows of
 * the paper's Table 1): the argmax over the D duration logits advances the
 * frame index; a blank advances it by at least one frame; a label with
 * duration 0 stays on the frame, at most max_symbols times in a row.
 *   durations_out [B, cap] or NULL: duration value of each label.
 * RNNT_ERR_VARIANT on an engine created with D == 0.
 */
int tdt_label_looping_decode(rnnt_engine *eng, const float *enc_out, const int32_t *enc_len,
                             int32_t B, int32_t T, int32_t max_symbols,
                             int32_t *tokens_out, int32_t *tok_len_out, int32_t cap,
                             int32_t *frames_out, float *logit_out, int32_t *durations_out,
                             rnnt_stream_t stream);

/*
 * The encoder-side joint projection alone (W_enc f + b_enc for every valid
 * frame), the part of joint() in Algorithm 1 that does not depend on the
 * prediction network and is therefore taken out of the loop.
 *   proj_out [B, T, J]; rows at t >= enc_len[b] are left untouched.
 */
int rnnt_encoder_projection(rnnt_engine *eng, const float *enc_out, const int32_t *enc_len,
                            int32_t B, int32_t T, float *proj_out, rnnt_stream_t stream);

/* Device status word of the last decode call (RNNT_DEV_* bits).  Waits for
 * the device.  *status_out is HOST memory. */
int rnnt_engine_status(rnnt_engine *eng, int32_t *status_out);

/* Work counters of the last decode call.  Waits for the device.  HOST out. */
int rnnt_engine_stats(rnnt_engine *eng, rnnt_stats *out);

/*
 * Tuning knobs, for measurement.  By default an engine holds one team layout
 * per range of launch sizes (1-2, 3-8, 9-16, ... utterances, up to
 * min(max_B, 128)), each with its own packed copy of the weights, and a
 * launch runs in the one for its size: a small batch is decoded the way an
 * engine created for that batch would decode it.  n_teams > 0 replaces them by
 * one layout of that many teams for every decoder and launch size; 0 keeps
 * the current layouts.  joint_groups (needs n_teams > 0): joint groups per team
 * in the label-looping calls, 0 or 1 = none; Algorithm 1 always runs plain
 * teams.  lookahead: frames examined per utterance per joint step (0 = default:
 * 8 in the label-looping calls, 16 when a call has one or two utterances; up
 * to 8 with at most 16 samples per step in Algorithm 1; 1 = one frame per
 * step).  search_steps: joint steps a search of
 * the label-looping calls may take before the team runs its next prediction
 * step for the rows that have their label (0 = chosen per call from the rows
 * per team, -1 = no limit).  None of the knobs changes a token.
 * Synchronous; repacks the weights when n_teams is given.  Returns
 * RNNT_ERR_SHAPE for values the engine cannot run (the work-groups do not
 * divide into the teams or groups, more than 16 utterances per team) and
 * RNNT_ERR_UNSUPPORTED when the layout does not fit the LDS; the layouts in
 * force stay as they were (after a lookahead that no layout fits: the default
 * layouts and lookahead).
 */
int rnnt_engine_configure(rnnt_engine *eng, int32_t n_teams, int32_t joint_groups,
                          int32_t lookahead, int32_t search_steps);

/*
 * Optional extra output of the decode calls that follow: logp_out, a DEVICE
 * buffer [B, cap] laid out like tokens_out, receives for every emitted label
 * its log-softmax value over the V1 token columns -- the value v that Algorithm 1
 * takes together with the argmax k from the log-probabilities of the joint
 * output (logit_out carries the maximum before the softmax).  The
 * log-sum-exp is fused into the argmax exchange of the joint step; nothing is
 * computed while no buffer is set.  NULL switches it off again.  The caller
 * owns the buffer and keeps it alive (cap as in the decode call) until the
 * calls that use it have finished.  Entries beyond tok_len are 0.
 */
int rnnt_engine_set_logp_output(rnnt_engine *eng, float *logp_out);

/*
 * Early return of finished utterances.  A batched decoder normally hands back
 * nothing before its slowest utterance is done (the paper's discussion of the
 * experiments names this as the price of batching); here utterances are
 * decoded independently inside one kernel, so each one's results are final
 * long before the call ends.
 *
 * done: [B] int32 the decode calls that follow write to, or NULL to switch the
 * flags off.  The caller sets done[0..B) to 0 before a call; the library only
 * ever stores 1.  As soon as utterance b has its last label, tok_len_out[b]
 * and the utterance's rows of every output buffer (fill beyond tok_len
 * included) are written and released at system scope, then done[b] = 1 is
 * stored.  A host thread that is to read results while the call still runs
 * passes pinned host memory (hipHostMalloc) for done and for the output
 * buffers, polls done[b] and reads row b once it sees 1; with device memory the
 * flags only order the outputs for other device-side readers.  When the call
 * has completed every flag is 1 unless the device status reports an aborted
 * call; the status word, not the flags, says whether results are valid.
 * The caller owns the array and keeps it alive until the calls have finished.
 */
int rnnt_engine_set_done_flags(rnnt_engine *eng, int32_t *done);

/*
 * How long the device-side waits of the decode calls that follow may last.  The
 * work-groups of a team wait for each other's results by polling; every such
 * wait gives up after `polls` repeated polls (one takes about a microsecond),
 * raises a flag that makes every other wait of the launch give up too, and the
 * call ends in the ordinary way with RNNT_DEV_ABORTED in the status word and
 * outputs that must not be used (Algorithm 1's loops have no such exit: this
 * is the bound that keeps a launch that did not get all its work-groups
 * resident, or a failing device, from hanging the stream).  polls = -1
 * restores the default, 2^22 (a few seconds); 0 lets a wait poll once, which
 * makes the first wait of a launch fail -- the way the tests reach the failure
 * path.  A later call on the engine starts clean.  RNNT_ERR_SHAPE for values
 * below -1 or above 2^32 - 1.
 */
int rnnt_engine_set_wait_limit(rnnt_engine *eng, int64_t polls);

/*
 * Phase timers of the last decode call, for libraries built with
 * -DRNNT_PROFILE (RNNT_PROFILE=1 in the environment of build.py): microseconds
 * rank 0 of `team` spent in each phase of the prediction and joint steps, as
 * many as n (at most 24) into the HOST array us_out.  The phases are listed in
 * bench.py (--phases).  An ordinary build returns RNNT_ERR_UNSUPPORTED.  Waits
 * for the device.
 */
int rnnt_engine_phase_timers(rnnt_engine *eng, int32_t team, double *us_out, int32_t n);

/*
 * Microbenchmarks of what bounds the decode path on the current device (not
 * part of the path; bench.py --probes prints them).  Synchronous; they
 * allocate and free their own buffers.
 *   rnnt_probe_stream    from_l2 = 1: every work-group reads, over and over, a
 *                        weight slice that stays in its XCD's L2, with the
 *                        decode kernel's access pattern; 0: every work-group
 *                        streams its own 8 MiB from HBM once.  GB/s over the
 *                        device and per compute unit.
 *   rnnt_probe_exchange  microseconds for one hand-over of a vector of `len`
 *                        floats inside teams of `team_size` work-groups (all
 *                        teams of the device at once): every work-group
 *                        writes its share and reads the whole vector, either
 *                        behind a counter barrier (tagged = 0) or as tagged
 *                        64-bit words that the readers poll (tagged = 1).
 *   rnnt_probe_mfma      fp32 matrix rate in TFLOP/s of the MFMA shape 4x4x1
 *                        in 16 blocks (shape 0, the decode kernel's) or
 *                        32x32x2 (shape 1, the projection kernel's).
 *   rnnt_probe_e4m3_widening  the bf16 (as 16-bit codes) that the conversion
 *                        used by the bfloat16 mode with e4m3-stored weights
 *                        makes of every e4m3 code under the scale operand
 *                        `scale` (the decode kernel passes a weight row's
 *                        power of two): bf16_out is a HOST array of 4 * 256
 *                        entries, [byte position in a word][code].
 *   rnnt_probe_e2m1_widening  the same for the 4-bit form: bf16_out is a HOST
 *                        array of 4 * 256 * 2 entries, [byte position][byte
 *                        value][code in the low, then the high nibble].
 * Return RNNT_OK or an RNNT_ERR_* code.
 */
int rnnt_probe_e4m3_widening(float scale, uint16_t *bf16_out);
int rnnt_probe_e2m1_widening(float scale, uint16_t *bf16_out);
int rnnt_probe_stream(int32_t from_l2, double *gbytes_per_s_out, double *per_cu_out);
int rnnt_probe_exchange(int32_t team_size, int32_t len, int32_t tagged, double *us_per_exchange_out);
int rnnt_probe_mfma(int32_t shape, double *tflops_out);

/* Text for a return code; for RNNT_ERR_HIP includes the last HIP error text. */
const char *rnnt_status_string(int code);

#ifdef __cplusplus
}
#endif
#endif /* RNNT_GREEDY_H */
