/*
 * dsla.h - C ABI of the MI355X (gfx950) dual-state linear attention (DSLA) layer forward.
 *
 * What the layer computes (paper Section 4.1 "Dual-State Linear Attention"), for every
 * (batch, head) pair independently, with row vectors q_t, k_t of length d_k and v_t, o_t
 * of length d_v, two d_k x d_v states S1 (history) and S2 (recency), forget gates
 * alpha1_t, alpha2_t in (0,1]^{d_k} (one value per token per feature, broadcast along
 * d_v) and a blend coefficient gamma:
 *
 *     S^i_t = diag(alpha^i_t) S^i_{t-1} + k_t^T v_t          i = 1, 2   (state update)
 *     o_t   = scale * q_t ( gamma S^1_t + (1 - gamma) S^2_t )            (read-out)
 *
 * The read-out uses the states after the update of the same token.  No feature map,
 * normaliser or output gate is applied.  Gates cross this boundary as natural
 * logarithms g^i_t = log alpha^i_t <= 0, never as alpha itself: a bf16 alpha close to one
 * would lose the decay rate.
 *
 * Conventions
 *  - Every pointer is a DEVICE pointer unless marked HOST.  The caller owns every
 *    buffer; the library allocates and frees no device memory and never synchronises:
 *    work is enqueued on the HIP stream passed as `stream` (a hipStream_t cast to void*,
 *    NULL = the default stream) and the call returns.
 *  - Layouts are contiguous with the last index fastest:
 *        q, k, g1, g2 : [B][T][H][d_k]        v, o : [B][T][H][d_v]
 *        S1, S2       : [B][H][d_k][d_v]  always fp32, updated in place
 *    (decode tensors are the same with the T index dropped).
 *    q, k, v, o have element type io_dtype; g1, g2 have element type gate_dtype.
 *    Pointers must be aligned to 16 bytes.
 *  - Errors: argument checks run on the host before anything is enqueued, so a call that
 *    returns an error other than DSLA_ERR_HIP has done nothing.  DSLA_ERR_HIP reports a
 *    failed launch (hipGetLastError text available through dsla_last_hip_error()).
 *  - Same inputs give bit-identical outputs (no atomics, fixed reduction order).
 *  - Supported shapes: d_k = d_v in {64, 128}; chunk in {0 (library default), 32, 64, 128};
 *    B, H, T >= 1 (T == 0 is accepted and does nothing).
 *  - Gate domain of dsla_prefill.  The prefill works through a sequence 32 tokens at a time and splits the decay
 *    between a query and a key of the same 32 tokens into a factor on each, both referred to the middle of those
 *    tokens' total decay; the factors are 2^(+-R/2) with R = the sum of |log2 alpha| over the 32 tokens, per
 *    feature.  They are exact while R <= 230, i.e. while the sum of |log alpha| over one aligned group of 32
 *    tokens stays below 159 for every feature (an average gate of 0.007 sustained over 32 tokens); gates of any
 *    strength are fine when they are not sustained, and nothing accumulates from one group of 32 to the next.
 *    Beyond that the result of the affected feature is undefined (inf or NaN may appear), and the kernels report
 *    it: if desc->status is not NULL they store DSLA_STATUS_GATE_DOMAIN there.  dsla_decode has no limit.
 */
#ifndef DSLA_H
#define DSLA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Exported with default visibility; everything else in the library is hidden. */
#define DSLA_API __attribute__((visibility("default")))

typedef enum {
    DSLA_OK = 0,
    DSLA_ERR_NULL = 1,        /* a required pointer is NULL                          */
    DSLA_ERR_SHAPE = 2,       /* non-positive size, misaligned pointer                */
    DSLA_ERR_UNSUPPORTED = 3, /* head size, chunk or dtype combination not built      */
    DSLA_ERR_WORKSPACE = 4,   /* workspace NULL or smaller than the query says        */
    DSLA_ERR_HIP = 5          /* a HIP call failed                                    */
} dsla_status;

typedef enum { DSLA_F32 = 0, DSLA_BF16 = 1 } dsla_dtype;

/*
 * What the gate tensors g1, g2 hold.  The paper describes the gates as driven by the data and produced by single linear
 * layers (Section 4.1, Section 5.3) without giving the map into (0,1]; this library takes the parametrisation
 * of the gated linear attention work the method extends: alpha = sigmoid(z)^(1/tau).
 *   DSLA_GATE_LOG    : g = log alpha <= 0, computed by the caller (any map into (0,1] can be used this way)
 *   DSLA_GATE_PREACT : g = z, the output of the gate projection; the kernels form
 *                      log alpha = -softplus(-z) / tau = (min(z,0) - log(1 + exp(-|z|))) / tau in fp32
 *                      themselves, which saves the caller one pass over both gate tensors
 */
typedef enum { DSLA_GATE_LOG = 0, DSLA_GATE_PREACT = 1 } dsla_gate_mode;

/* Layer descriptor (HOST memory, read during the call only). */
typedef struct {
    int32_t B;          /* sequences in the batch                                       */
    int32_t H;          /* heads                                                        */
    int32_t d_k;        /* width of q, k and the gates; rows of a state                 */
    int32_t d_v;        /* width of v, o; columns of a state                            */
    int32_t chunk;      /* prefill chunk length C; 0 = library default; decode ignores  */
    int32_t segments;   /* prefill: 0 = choose automatically; > 0 = split every sequence
                           into this many segments processed in parallel (tuning/tests);
                           the result does not depend on it beyond rounding             */
    int32_t io_dtype;   /* dsla_dtype of q, k, v, o                                     */
    int32_t gate_dtype; /* dsla_dtype of g1, g2                                         */
    int32_t gate_mode;  /* dsla_gate_mode: what g1, g2 hold                             */
    int32_t zero_init;  /* prefill: nonzero = the states are zero before the first token (dsla_state_init folded
                           into the call): S1, S2 are not read, only written.  decode ignores it   */
    float tau;          /* DSLA_GATE_PREACT: temperature, finite and > 0 (16 in the gated linear attention
                           work; 1 = plain sigmoid); ignored for DSLA_GATE_LOG          */
    float gamma;        /* blend coefficient of the layer (read-out equation); any real */
    float scale;        /* multiplies q (e.g. d_k^-1/2); 1.0 = the paper's plain form   */
    const float *gamma_per_head; /* optional DEVICE array [H] overriding gamma; or NULL */
    int32_t *status;    /* optional DEVICE word or NULL.  The prefill kernels store DSLA_STATUS_GATE_DOMAIN in it
                           when a group of 32 tokens leaves the gate domain described above; they never clear it
                           (the caller zeroes it and reads it back when it wants to know)                     */
} dsla_desc;

#define DSLA_STATUS_GATE_DOMAIN 1

/*
 * dsla_state_init - set both states to zero, the initial condition implied by the
 * unrolled form of Section 4.1 (no term from before the first token).
 * S1, S2: [B][H][d_k][d_v] fp32, written.
 */
DSLA_API dsla_status dsla_state_init(const dsla_desc *desc, float *S1, float *S2, void *stream);

/*
 * dsla_prefill_workspace_bytes - size in bytes of the scratch buffer dsla_prefill needs
 * for this descriptor and sequence length (0 when none is needed).  Returns 0 for an
 * invalid descriptor as well; dsla_prefill reports the actual error.
 */
DSLA_API size_t dsla_prefill_workspace_bytes(const dsla_desc *desc, int64_t T);

/*
 * dsla_prefill - the layer over T tokens per sequence, in chunks of C tokens: within a
 * chunk the state update and read-out of Section 4.1 are evaluated as dense
 * contractions, and the two states are carried from chunk to chunk.  The result equals
 * the token-by-token recurrence up to rounding for every T >= 1 (a ragged last chunk is
 * masked).
 *
 *   q, k, v, g1, g2 : inputs, layouts above          o : output, [B][T][H][d_v]
 *   S1, S2          : states before the first token on entry, after the last on return;
 *                     calling again with the next T' tokens continues the sequence
 *   workspace       : at least dsla_prefill_workspace_bytes(desc, T) bytes, 256-byte
 *                     aligned; contents are scratch (undefined before and after)
 * Built combinations: d in {64, 128}, chunk in {32, 64, 128}, io and gate dtype bf16 or f32;
 *                     chunk = 0 selects 64.  The chunk length is the granularity of the internal
 *                     split of long sequences into segments (a segment is a whole number of
 *                     chunks); the contractions themselves always cover 32 tokens.  The result
 *                     does not depend on it beyond rounding.
 * io f32 uses fp32 arithmetic throughout; io bf16 rounds contraction operands to bf16
 * and accumulates in fp32; states are fp32 in both.
 */
DSLA_API dsla_status dsla_prefill(const dsla_desc *desc, int64_t T,
                         const void *q, const void *k, const void *v,
                         const void *g1, const void *g2,
                         float *S1, float *S2, void *o,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * dsla_prefill_static_ws - dsla_prefill with the scratch buffer built into the library, for callers that cannot
 * allocate device memory or size a workspace at the point of the call: code under HIP graph capture, tight
 * serving loops, harnesses that forbid allocation.  Same arguments as dsla_prefill without the workspace; same
 * kernels, same results.  The scratch is a fixed array of DSLA_STATIC_WORKSPACE_BYTES bytes in the library's
 * device code, one copy per GPU, held from the moment the library is loaded on that GPU until the process ends.
 *   - The call allocates and frees nothing.  The first call on a device looks up the array's address there.
 *   - The device current at the time of the call must be the one `stream` and the buffers belong to.
 *   - A plan that needs more than DSLA_STATIC_WORKSPACE_BYTES (see dsla_prefill_workspace_bytes) is rejected with
 *     DSLA_ERR_WORKSPACE before anything is enqueued; the headline shape (B = 1, H = 32, d = 128, T = 16384) needs
 *     32.2 MiB, and no plan the library makes itself at d = 128 needs more than 48.3 MiB (B H = 128).
 *   - All calls on one GPU share the array: calls that may overlap there (different streams, different threads)
 *     race and must be ordered by the caller.  Nothing in the array has to start at zero and nothing in it outlives
 *     a call: every slot is written by the call before it is read.
 */
#define DSLA_STATIC_WORKSPACE_BYTES ((size_t)64 << 20)
DSLA_API dsla_status dsla_prefill_static_ws(const dsla_desc *desc, int64_t T,
                                   const void *q, const void *k, const void *v,
                                   const void *g1, const void *g2,
                                   float *S1, float *S2, void *o, void *stream);

/*
 * dsla_prefill_varlen - dsla_prefill for a batch of sequences of different lengths packed back to back along
 * the token axis, with each sequence's states at a caller-chosen place in a pool of states: the prefill half
 * of the mixed prefill/decode batches of the paper's serving system (Section 4.5 and the appendix "Serving of Mixed Batch"),
 * where requests of different prompt lengths are processed together and each keeps its own pair of states.
 * Every sequence is an independent instance of the recurrence of Section 4.1.
 *
 *   desc->B        : number of sequences this call processes
 *   total_T        : tokens in the packed batch (cu_seqlens' last entry); at most 2^31 - 1
 *   max_T          : an upper bound of the sequence lengths, max_T <= total_T.  It is used for planning only;
 *                    a sequence longer than max_T is NOT processed correctly (the library cannot see the
 *                    lengths without synchronising)
 *   cu_seqlens     : DEVICE int32 [B + 1], non-decreasing, cu_seqlens[0] >= 0: sequence b is the tokens
 *                    cu_seqlens[b] .. cu_seqlens[b+1] - 1.  A sequence of length 0 is legal: its states stay
 *                    as they are and it has no output rows
 *   seq_index      : DEVICE int32 [B] or NULL.  Which of the packed sequences take part: entry b of this call is
 *                    sequence seq_index[b] of cu_seqlens (which then has more than B + 1 entries); NULL = the
 *                    first B, in order.  This is how the requests of a mixed batch that use the DSLA form of
 *                    a layer are processed where they lie, without a split into a sub-batch and a merge
 *                    afterwards (Section 4.5): the rows of the other sequences are neither read nor written.
 *                    total_T stays the size of the whole packed batch, max_T bounds the participating lengths
 *   state_slot     : DEVICE int32 [B] or NULL.  The states of sequence b are entry state_slot[b] of S1, S2
 *                    ([n_slots][H][d_k][d_v], n_slots known to the caller only); NULL = entry b.  Values must
 *                    be valid and distinct (two sequences on one entry race); other entries are not touched
 *   q, k, g1, g2   : [total_T][H][d_k]      v, o : [total_T][H][d_v]
 *   workspace      : at least dsla_prefill_varlen_workspace_bytes(desc, total_T, max_T) bytes, 256-byte aligned
 * Everything else (chunking, gate domain, dtypes, in-place continuation of the states) is as for dsla_prefill.
 * desc->segments > 0 cuts a sequence of max_T tokens into that many segments; shorter sequences use the first
 * few of them.
 */
DSLA_API size_t dsla_prefill_varlen_workspace_bytes(const dsla_desc *desc, int64_t total_T, int64_t max_T);
DSLA_API dsla_status dsla_prefill_varlen(const dsla_desc *desc, int64_t total_T, int64_t max_T,
                                const int32_t *cu_seqlens, const int32_t *seq_index, const int32_t *state_slot,
                                const void *q, const void *k, const void *v,
                                const void *g1, const void *g2,
                                float *S1, float *S2, void *o,
                                void *workspace, size_t workspace_bytes, void *stream);

/*
 * dsla_decode - one token per sequence: the state update and read-out of Section 4.1
 * applied once, fused so that each state is read from and written to memory exactly once.
 *   q, k, g1, g2 : [B][H][d_k]     v : [B][H][d_v]     o : [B][H][d_v] (written)
 *   S1, S2       : updated in place
 */
DSLA_API dsla_status dsla_decode(const dsla_desc *desc,
                        const void *q, const void *k, const void *v,
                        const void *g1, const void *g2,
                        float *S1, float *S2, void *o, void *stream);

/*
 * dsla_decode_slots - dsla_decode with the states of sequence b at entry state_slot[b] (DEVICE int32 [B], valid
 * and distinct) of S1, S2 = [n_slots][H][d_k][d_v]: the decode half of a mixed batch, where the requests that
 * are decoding in this step are a changing subset of the requests whose states are resident (Section 4.5).
 * Entries not named are not touched.  row_index (DEVICE int32 [B], distinct, or NULL = row b): the token of
 * sequence b is row row_index[b] of q, k, v, g1, g2 ([rows][H][d]) and its output goes to the same row of o, so
 * the DSLA requests of a larger batch are served in place (no split and merge, Section 4.5); other rows of o
 * are not written.
 */
DSLA_API dsla_status dsla_decode_slots(const dsla_desc *desc,
                              const void *q, const void *k, const void *v,
                              const void *g1, const void *g2,
                              const int32_t *row_index, const int32_t *state_slot,
                              float *S1, float *S2, void *o, void *stream);

/*
 * More than two states, the general outer-product gate, grouped key/value heads.
 *
 * The background section on gated linear attention writes the forget gate of a state as a d_k x d_v matrix formed
 * as the outer product of two vectors, G_t = alpha_t^T beta_t; Section 4.2 ("Why Two States Suffice?") and the
 * ablation over the number of states in Section 5.5 consider the same layer with 1, 2, 4 or 8 states, each with its
 * own gate; the Llama-3 teacher of Section 5.5 has grouped key/value heads.  For state n = 0 .. n_states - 1:
 *     S^n_t[d][j] = alpha^n_t[d] beta^n_t[j] S^n_{t-1}[d][j] + k_t[d] v_t[j]
 *     o_t         = scale * q_t * sum_n w_n S^n_t
 * The paper prints the blend for two states only (gamma, 1 - gamma); one real coefficient per state is the reading
 * taken for N states, and (gamma, 1 - gamma) is its case N = 2.  desc->gamma and desc->gamma_per_head are not used
 * by these calls; everything else in the descriptor means what it means for dsla_prefill / dsla_decode
 * (gate_mode applies to alpha and beta alike).
 *   q, g_alpha[n]     : [B][T][H][d_k]      g_beta[n] : [B][T][H][d_v]      o : [B][T][H][d_v]
 *   k                 : [B][T][H_kv][d_k]   v         : [B][T][H_kv][d_v]   head h reads key/value head h / (H / H_kv)
 *   S[n]              : [B][H][d_k][d_v] fp32, one pair of pointers per state, every query head keeps its own states
 * (decode: the same without the T index).
 */
#define DSLA_MAX_STATES 8
typedef struct {
    int32_t n_states;              /* 1 .. DSLA_MAX_STATES                                                      */
    int32_t H_kv;                  /* key/value heads, a divisor of desc->H; 0 = desc->H                        */
    const void *const *g_alpha;    /* HOST array [n_states] of DEVICE pointers: log alpha^n (or pre-activations) */
    const void *const *g_beta;     /* HOST array [n_states] of DEVICE pointers (entries may be NULL), or NULL:
                                      log beta^n; NULL means beta^n = 1                                         */
    float *const *S;               /* HOST array [n_states] of DEVICE pointers, updated in place                */
    const float *weights;          /* HOST array [n_states]: blend coefficients w_n of the layer                */
    const float *weights_per_head; /* optional DEVICE array [n_states][H] overriding weights; or NULL           */
} dsla_multi;

/*
 * dsla_decode_multi - one token per sequence for a layer described by desc and multi; every state is read once and
 * written once.  All of n_states, both gate vectors and H_kv are supported.
 */
DSLA_API dsla_status dsla_decode_multi(const dsla_desc *desc, const dsla_multi *multi,
                              const void *q, const void *k, const void *v, void *o, void *stream);

/*
 * dsla_prefill_multi - T tokens per sequence for a layer described by desc and multi.  The states without a beta
 * gate are taken two at a time through the kernels of dsla_prefill (an odd one out runs with an idle partner); a
 * state with a beta gate runs on its own in a mode of the same kernels that splits the decay along the columns of
 * the state between the values on the way in and the output on the way out, as the decay along the rows is split
 * between keys and queries (the gate domain of dsla_prefill then holds for beta as for alpha).  Every launch after
 * the first adds its share to o; grouped key/value heads are an index map inside the kernels.
 * workspace: at least dsla_prefill_multi_workspace_bytes(desc, multi, T) bytes, 256-byte aligned.
 */
DSLA_API size_t dsla_prefill_multi_workspace_bytes(const dsla_desc *desc, const dsla_multi *multi, int64_t T);
DSLA_API dsla_status dsla_prefill_multi(const dsla_desc *desc, const dsla_multi *multi, int64_t T,
                               const void *q, const void *k, const void *v, void *o,
                               void *workspace, size_t workspace_bytes, void *stream);

/*
 * dsla_attention_entropy - the sensitivity signal of Section 4.3 ("Layer Ranking via Sensitivity") for a
 * softmax-attention layer: for every (batch, head), the attention row of the final query over the T keys,
 * A_i = softmax_i(scale * q_T . k_i), and its entropy.  The paper's display shows sum_i A_i log A_i; this returns
 * the entropy proper, H = -sum_i A_i log A_i >= 0 (natural logarithm), the negative of that sum: low values mean
 * attention concentrated on few tokens, which the paper reads as a layer that loses little when converted.
 * Averaging over heads and ranking the layers is left to the caller.
 *   B, H, d     : batch, heads, head size (d in {64, 128});  T >= 1 keys per sequence
 *   io_dtype    : dsla_dtype of q_last and k
 *   q_last      : [B][H][d], the query of the last position      k : [B][T][H][d]
 *   entropy     : [B][H] fp32, written
 *   workspace   : at least dsla_attention_entropy_workspace_bytes(B, H, d, T) bytes, 16-byte aligned (0 bytes when
 *                 there are enough (batch, head) pairs to fill the device; then it may be NULL)
 * Arithmetic is fp32; one pass over the keys.  Errors and stream semantics as for the other entry points.
 */
DSLA_API size_t dsla_attention_entropy_workspace_bytes(int32_t B, int32_t H, int32_t d, int64_t T);
DSLA_API dsla_status dsla_attention_entropy(int32_t B, int32_t H, int32_t d, int64_t T, int32_t io_dtype, float scale,
                                   const void *q_last, const void *k, float *entropy,
                                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * dsla_attention_decode - one decode step of a softmax-attention layer that has NOT been converted: one query per
 * (batch, head) against the T cached keys and values of its sequence (the current token included),
 *     o = sum_i softmax_i(scale * q . k_i) v_i .
 * This is what the paper's serving system runs beside the DSLA layers of a partly converted model (Section 4.3) and
 * what the constant-cost DSLA decode step is measured against (Section 5.3): its traffic is the whole cache, 4 d T
 * bytes per head in bf16, against two fixed states.
 *   B, H, d     : batch, heads, head size (d in {64, 128});  T >= 1 positions the cache of a sequence can hold
 *   io_dtype    : dsla_dtype of q, k, v, o
 *   q           : [B][H][d]      k, v : [B][T][H][d]      o : [B][H][d], written
 *   seq_lens    : DEVICE int32 [B] or NULL.  Positions sequence b has filled, 1 <= seq_lens[b] <= T (requests of a
 *                 batch are at different context lengths); only those are read.  NULL = T for every sequence
 *   workspace   : at least dsla_attention_decode_workspace_bytes(B, H, d, T) bytes, 16-byte aligned (0 bytes when
 *                 there are enough (batch, head) pairs to fill the device; then it may be NULL)
 * fp32 arithmetic, one pass over keys and values.  Errors and stream semantics as for the other entry points.
 */
DSLA_API size_t dsla_attention_decode_workspace_bytes(int32_t B, int32_t H, int32_t d, int64_t T);
DSLA_API dsla_status dsla_attention_decode(int32_t B, int32_t H, int32_t d, int64_t T, int32_t io_dtype, float scale,
                                  const void *q, const void *k, const void *v, const int32_t *seq_lens, void *o,
                                  void *workspace, size_t workspace_bytes, void *stream);

/*
 * dsla_project - the projections in front of a DSLA layer as one MFMA GEMM (Section 5.3: the gates come from single
 * linear layers; appendix on training details: q, k, v reuse the teacher's projections, the history gate's weight starts
 * near the identity, the recency gate's from a normal distribution, biases zero).  From the layer input x and the
 * stacked weights it writes n_out tensors - typically q, k, v and the pre-activations of the two gates - each in the
 * layout the prefill reads, so that dsla_prefill with gate_mode = DSLA_GATE_PREACT runs on them as they are:
 *     out_j[m][c] = sum_k x[m][k] W[j * width + c][k] (+ bias[j * width + c]),     j = 0 .. n_out - 1
 *   M          : rows of x = batch * tokens (>= 1)
 *   K          : model width, a multiple of 32 and at most 2^21 (a multiple of 128 takes the faster kernel: 256 x 256
 *                output tiles instead of 128 x 128)
 *   n_out      : 1 .. DSLA_MAX_PROJECTIONS output tensors, each `width` = H * d wide, a multiple of 128
 *   x          : [M][K] bf16          W : [n_out * width][K] bf16, row-major (a linear layer's weight)
 *   bias       : [n_out * width] fp32 or NULL
 *   outs       : HOST array [n_out] of DEVICE pointers, each [M][width] bf16, written
 * bf16 operands, fp32 accumulation; no workspace.  Errors and stream semantics as for the other calls.
 */
#define DSLA_MAX_PROJECTIONS 8
DSLA_API dsla_status dsla_project(int64_t M, int32_t K, int32_t n_out, int32_t width,
                         const void *x, const void *W, const float *bias, void *const *outs, void *stream);

/*
 * dsla_attention_prefill - causal softmax attention over a whole prompt: the prefill of a layer that has NOT been
 * converted, which a partly converted model runs beside its DSLA layers (Section 4.3) and whose quadratic cost the
 * linear-time DSLA prefill is measured against (Section 5.3):
 *     o_t = sum_{i <= t} softmax_{i <= t}(scale * q_t . k_i) v_i .
 *   B, H, d  : batch, heads, head size (d in {64, 128});  T >= 1 tokens per sequence, one sequence's tensor
 *              (T * H * d * 2 bytes) below 4 GiB, else DSLA_ERR_SHAPE
 *   io_dtype : DSLA_BF16 only (bf16 operands on MFMA, fp32 accumulation and softmax statistics); DSLA_F32 is
 *              DSLA_ERR_UNSUPPORTED
 *   q, k, v  : [B][T][H][d]      o : [B][T][H][d], written
 * One pass over the keys with a running maximum; no workspace.  Errors and stream semantics as for the other calls.
 */
DSLA_API dsla_status dsla_attention_prefill(int32_t B, int32_t H, int32_t d, int64_t T, int32_t io_dtype, float scale,
                                   const void *q, const void *k, const void *v, void *o, void *stream);

/*
 * Host-side conversion logic (paper Section 4.3 "Adaptive Layer-wise Conversion").  Plain host functions, HOST
 * pointers, no device work: they decide which layers of a model run in DSLA form for a request; the calls above
 * then run those layers (the entropy that ranks them comes from dsla_attention_entropy).
 *
 * dsla_rank_layers          - "Layer Ranking via Sensitivity": order[0 .. n_layers) = the layer indices in ascending
 *                             order of sensitivity (the layer that loses least when converted first); equal scores
 *                             keep the lower index first.  A NaN score is DSLA_ERR_SHAPE.
 * dsla_max_conversion_rate  - the table of the trace replay (Section 5.4): the largest fraction of layers converted
 *                             for a prompt of that many tokens: below 2048 12.5 %, below 4096 25 %, below 8192
 *                             37.5 %, else 50 % (the paper's "2k", "4k", "8k" read as multiples of 1024).
 * dsla_kv_cache_bytes       - Section 5.3: 2 * n_layers * batch * context * heads * d_head * bytes_per_element
 *                             (-1 for a negative argument).
 * dsla_conversion_plan      - "Adaptive Conversion Logic": when memory_used exceeds memory_threshold, convert layers
 *                             from the least sensitive end of `order` (a permutation of the layers, as
 *                             dsla_rank_layers returns it), each conversion trading kv_bytes_per_layer for
 *                             state_bytes_per_layer, until use falls to the threshold (memory relief) or
 *                             floor(max_rate * n_layers) layers are converted (the quality limit, as the cap of the
 *                             trace replay).  converted[layer] (HOST, n_layers bytes) = 1 for a converted layer;
 *                             *n_converted their number; *memory_after and *reason (DSLA_PLAN_*) optional.
 */
#define DSLA_PLAN_NO_PRESSURE 0
#define DSLA_PLAN_MEMORY_RELIEF 1
#define DSLA_PLAN_QUALITY_LIMIT 2
#define DSLA_PLAN_ALL_CONVERTED 3
DSLA_API dsla_status dsla_rank_layers(int32_t n_layers, const float *sensitivity, int32_t *order);
DSLA_API float dsla_max_conversion_rate(int64_t prompt_len);
DSLA_API int64_t dsla_kv_cache_bytes(int32_t n_layers, int64_t batch, int64_t context, int32_t heads, int32_t d_head,
                            int32_t bytes_per_element);
DSLA_API dsla_status dsla_conversion_plan(int32_t n_layers, const int32_t *order, int64_t memory_used,
                                 int64_t memory_threshold, int64_t kv_bytes_per_layer, int64_t state_bytes_per_layer,
                                 float max_rate, uint8_t *converted, int32_t *n_converted, int64_t *memory_after,
                                 int32_t *reason);

/* Text for a status code (static storage). */
DSLA_API const char *dsla_status_string(dsla_status s);

/* Text of the last HIP error seen by this thread's calls into the library (static). */
DSLA_API const char *dsla_last_hip_error(void);

/*
 * Kernel timing for benchmarks.  While enabled, every kernel the library launches carries
 * two HIP events in its dispatch (hipExtLaunchKernelGGL: the start and the end of the kernel
 * are stamped by the dispatch itself, on the launch stream, and no event packet of its own
 * delays the launch that follows; events come from a pool created by dsla_profile_enable,
 * so the launch path still allocates nothing).
 * Kernel ids: 0 state_init, 1 prefill_segment_state, 2 prefill_segment_scan,
 * 3 prefill_chunk_loop, 4 decode, 5 prefill_segment_list (packed sequences only), 6 attention_entropy,
 * 7 attention_decode (each with its merge kernel), 8 decode_multi, 9 attention_prefill, 10 project.
 */
#define DSLA_KERNEL_STATE_INIT 0
#define DSLA_KERNEL_PREFILL_SEGMENT_STATE 1
#define DSLA_KERNEL_PREFILL_SEGMENT_SCAN 2
#define DSLA_KERNEL_PREFILL_CHUNK_LOOP 3
#define DSLA_KERNEL_DECODE 4
#define DSLA_KERNEL_PREFILL_SEGMENT_LIST 5
#define DSLA_KERNEL_ATTENTION_ENTROPY 6
#define DSLA_KERNEL_ATTENTION_DECODE 7
#define DSLA_KERNEL_DECODE_MULTI 8
#define DSLA_KERNEL_ATTENTION_PREFILL 9
#define DSLA_KERNEL_PROJECT 10
#define DSLA_KERNEL_COUNT 11

/* enable != 0: create the event pool (max_records launches can be recorded between two
 * collects) and start recording; enable == 0: stop and destroy the pool. */
DSLA_API dsla_status dsla_profile_enable(int enable, int max_records);
/* Waits for the recorded events, adds up elapsed milliseconds and launch counts per
 * kernel id into the HOST arrays total_ms[DSLA_KERNEL_COUNT], launches[DSLA_KERNEL_COUNT],
 * and clears the records. */
DSLA_API dsla_status dsla_profile_collect(double *total_ms, int64_t *launches);

#ifdef __cplusplus
}
#endif
#endif /* DSLA_H */
