/*
 * sp.h -- C ABI of the MI355X (gfx950) K-student forward of Student Parallelism.
 *
 * The library runs the inference hot path of the paper's method: a group of K
 * shallow BERT-like student encoders, all evaluated on the same padding-free
 * batch of variable-length sequences, whose per-student classifier outputs are
 * summed over the first k_active students (boosting ensemble, Section 3.1 Eq. 1;
 * classifier on the ensembled representation, Section 3.2 Algorithm 2 lines 5-6;
 * students are dropped from the tail at run time, Section 3.2 / Section 3.3.1).
 *
 * Conventions for every entry point
 *   - return value 0 on success, a negative SP_E* code otherwise; no exception,
 *     abort or global state crosses this boundary;
 *   - "host" / "device" on a pointer says where the memory lives; the library
 *     never takes ownership of caller memory and never frees it;
 *   - all device memory (weight arena, workspace, inputs, outputs) is allocated
 *     by the caller; sp_forward itself allocates nothing and does not
 *     synchronise with the host: it enqueues kernels on the given stream and
 *     returns.
 */
#ifndef SP_H_
#define SP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    SP_OK = 0,
    SP_EINVAL = -1,   /* null or misaligned pointer, malformed config */
    SP_ESHAPE = -2,   /* batch < 1, total_tokens < batch, max_seqlen > max_pos, unsupported head width ... */
    SP_EKACTIVE = -3, /* k_active outside 1..K */
    SP_ENOMEM = -4,   /* weight blob, arena or workspace smaller than required */
    SP_EHIP = -5,     /* a HIP runtime call failed */
    /* -6, -7: the length-aware buffer's codes (sp_dispatch.h) */
    SP_ETOOBIG = -8   /* sp_forward_static: the call needs more workspace than the library's static array holds */
};

enum { SP_DTYPE_FP32 = 0, SP_DTYPE_BF16 = 1, SP_DTYPE_FP8 = 2 };

/* Shape of the student group.  All students share one architecture (Section 3.1:
 * homogeneous students so that none is a straggler). */
typedef struct {
    int32_t K;        /* students in the group, index = training order */
    int32_t layers;   /* transformer layers per student */
    int32_t hidden;   /* H */
    int32_t heads;    /* A; head width H/A must be 64 */
    int32_t ffn;      /* F */
    int32_t vocab;    /* V */
    int32_t max_pos;  /* P: longest sequence a student can take */
    int32_t classes;  /* C, 1..16 */
    int32_t dtype;    /* SP_DTYPE_FP32: fp32 storage and arithmetic;
                         SP_DTYPE_BF16: bf16 weights and activations, fp32 accumulation,
                         LayerNorm statistics, softmax, GELU, pooling and logits;
                         SP_DTYPE_FP8: quantised students (Section 2, Related Work: the method is orthogonal
                         to quantisation, every student can be quantised).  The bf16 path, except that in calls
                         of >= 2048 token rows the four projections (query/key/value, attention output, FFN
                         up, FFN down) of every all-token layer run on fp8 (OCP e4m3) operands: weights quantised at load with one
                         fp32 scale per output feature (max |w| -> 448), activations quantised by the kernel
                         that produces them as e4m3(16 * value) (one fixed power-of-two scale per tensor; the
                         FFN activations exist only in fp8), fp32 accumulation, same epilogues.  Attention
                         itself, the first-token last layer, the head, all smaller calls, and students whose
                         hidden or FFN width is not a multiple of 256 stay bf16 (the arena keeps both copies
                         of the four matrices). */
    float ln_eps;     /* LayerNorm epsilon (BERT: 1e-12) */
    int32_t last_layer_all_tokens;
                      /* Only the first token of each sequence feeds the head (the pooled representation of
                         Section 3.1), so in the last layer every other row is dead work.  0 (default): bf16
                         calls with >= 1024 tokens compute the last layer for the first-token rows only:
                         their queries are folded through the key projection, the other tokens' keys and
                         values are never formed, and the output projection, FFN and LayerNorms run on
                         `batch` rows (same function; the rounding points of attention differ); bf16 calls
                         of up to four sequences (and fewer than 1024 tokens) compute the last layer's attention for every
                         token and everything after it for the first-token rows only.  1: every token goes
                         through the whole last layer (what a stock BERT does; the fp32 path always does). */
    int32_t single_stream;
                      /* 0 (default): a call with >= 2048 tokens and k_active >= 2 runs the active students
                         as two groups side by side, the second on a stream the model owns, forked from and
                         joined to the caller's stream with events (the call stays asynchronous and can be
                         captured in a graph; the logits are bit-identical to the single-stream result).
                         1: everything is enqueued on the caller's stream. */
} sp_config;

typedef struct sp_model sp_model; /* opaque host-side handle */

/* Canonical host weight blob: float32, per student m = 0..K-1 in this order
 *   tok_emb[V][H] pos_emb[P][H] emb_ln_g[H] emb_ln_b[H]
 *   per layer: Wq[H][H] bq[H] Wk[H][H] bk[H] Wv[H][H] bv[H] Wo[H][H] bo[H]
 *              ln1_g[H] ln1_b[H] W1[H][F] b1[F] W2[F][H] b2[H] ln2_g[H] ln2_b[H]
 *   Wp[H][H] bp[H] Wc[H][C] bc[C]
 * every matrix [in][out] row-major.  The ensemble multipliers alpha of Eq. 1
 * are expected folded into Wc (and the shared classifier bias placed in
 * student 0's bc): a linear classifier on sum_m alpha_m p_m equals the sum of
 * per-student heads alpha_m Wc.  Returns the number of floats in the blob, 0
 * for a malformed config. */
size_t sp_blob_floats(const sp_config* cfg);

/* Device bytes needed for the repacked weights of the whole group. */
size_t sp_arena_bytes(const sp_config* cfg);

/* Device bytes of workspace sp_forward needs for a call with at most
 * max_tokens packed tokens and max_batch sequences (monotone in both). */
size_t sp_workspace_bytes(const sp_config* cfg, int32_t max_tokens, int32_t max_batch);

/* Load the group (Algorithm 1 leaves the students in training order; that order
 * is kept: student 0 is the one that survives every pruning).
 *   host_weights  host, read-only, nfloats float32 values in blob order
 *   device_arena  device, caller-allocated, >= sp_arena_bytes, 256-byte aligned;
 *                 filled here (bf16 mode rounds to nearest even once) and
 *                 referenced by the returned handle until sp_free
 *   hip_stream    hipStream_t (or NULL for the default stream) the upload is
 *                 ordered on; the call returns after the upload has completed
 *   out           receives the handle
 * Errors: SP_EINVAL, SP_ESHAPE (config the kernels do not support), SP_ENOMEM
 * (nfloats or arena_bytes too small), SP_EHIP. */
int sp_load_students(const sp_config* cfg, const float* host_weights, size_t nfloats,
                     void* device_arena, size_t arena_bytes, void* hip_stream, sp_model** out);

/* One forward pass (Section 3.3: one batch of individual samples and the current
 * student number in, one prediction per sample out).
 *   token_ids    device int32 [total_tokens]: the sequences back to back, no
 *                padding; values in 0..V-1
 *   cu_seqlens   device int32 [batch+1]: cu[0] = 0, cu[b+1] - cu[b] = length of
 *                sequence b (>= 1), cu[batch] = total_tokens.  The first token
 *                of a sequence is the one whose final state is pooled; a token's
 *                position is its index inside its own sequence.
 *   max_seqlen   upper bound on every sequence length in this call, <= P
 *   k_active     1..K: only students 0..k_active-1 are evaluated and summed,
 *                in that order, in fp32
 *   workspace    device, 256-byte aligned, >= sp_workspace_bytes(cfg,
 *                total_tokens, batch); contents undefined afterwards; calls
 *                that may overlap in time need separate workspaces
 *   logits_out   device float32 [batch][classes] row-major, overwritten (written once, never read: pinned host memory
 *                that the device can address will do as well, through its device pointer)
 *   hip_stream   hipStream_t (or NULL); kernels are enqueued there
 * Contents of token_ids / cu_seqlens are not inspected on the host (that
 * would need a synchronisation): ids outside the vocabulary or inconsistent
 * offsets are the caller's error; ids are clamped into the table and lengths
 * into 1..max_seqlen on the device so that no access leaves its buffer.
 * Errors: SP_EINVAL, SP_ESHAPE, SP_EKACTIVE, SP_ENOMEM, SP_EHIP (launch failure). */
int sp_forward(const sp_model* model, const int32_t* token_ids, const int32_t* cu_seqlens,
               int32_t batch, int32_t total_tokens, int32_t max_seqlen, int32_t k_active,
               void* workspace, size_t workspace_bytes, float* logits_out, void* hip_stream);

/* sp_forward for callers that cannot allocate device memory and have no workspace to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The workspace is a static device array inside the
 * library, SP_STATIC_SCRATCH_MIB MiB per GPU (part of the library's device image: each GPU the library runs on holds
 * it until the process ends); the call itself allocates nothing, frees nothing and calls no allocating routine.  It
 * enqueues exactly the kernels sp_forward would, so the logits are bit-identical to sp_forward's.
 *   - the model's GPU must be the current device;
 *   - arguments as for sp_forward, without the workspace; inputs and logits_out are still the caller's;
 *   - a call that needs more than the array holds (sp_workspace_bytes(cfg, total_tokens, batch) >
 *     sp_static_scratch_bytes(): for the 8-student hidden-768 group that is any call of more than 256 tokens)
 *     returns SP_ETOOBIG and enqueues nothing;
 *   - every call on a GPU, from any model, stream or thread, uses that GPU's one array, which keeps the previous
 *     call's contents (nothing in it has to start at zero: a forward writes every row it reads).  Calls that can
 *     overlap in time on one GPU race on it: order them (one stream, or events), or use sp_forward with a
 *     workspace per call.
 * Errors: those of sp_forward, and SP_ETOOBIG. */
#define SP_STATIC_SCRATCH_MIB 64
size_t sp_static_scratch_bytes(void);
int sp_forward_static(const sp_model* model, const int32_t* token_ids, const int32_t* cu_seqlens,
                      int32_t batch, int32_t total_tokens, int32_t max_seqlen, int32_t k_active,
                      float* logits_out, void* hip_stream);

/* Releases the host handle only; the arena stays the caller's. */
void sp_free(sp_model* model);

/* Static description of an error code. */
const char* sp_strerror(int code);

/* Padding-free packing offsets on the host (Section 3.3.2 and Table 4 "with
 * padding" motivate batches without padding): cu[0] = 0, cu[i+1] = cu[i] +
 * lengths[i].  lengths_host [batch], cu_seqlens_host [batch+1].  SP_ESHAPE if a
 * length is < 1 or the total exceeds INT32_MAX. */
int sp_pack(const int32_t* lengths_host, int32_t batch, int32_t* cu_seqlens_host);

/* Contents check of the device-resident inputs of a forward, for callers that cannot vouch for them (sp_forward
 * itself never inspects them: that would need a synchronisation; it clamps on the device instead).  One small kernel
 * on hip_stream, then a synchronous copy of one word: this call blocks.  *problems_host receives a bit set:
 *   SP_BAD_ID       a token id outside 0..V-1
 *   SP_BAD_CU0      cu_seqlens[0] != 0
 *   SP_BAD_ORDER    an offset not larger than its predecessor (a sequence of length < 1)
 *   SP_BAD_LENGTH   a sequence longer than max_seqlen
 *   SP_BAD_TOTAL    cu_seqlens[batch] != total_tokens
 * scratch: device, >= 4 bytes, 4-byte aligned (any part of a workspace will do; its first word is overwritten).
 * Errors: SP_EINVAL, SP_ESHAPE (batch < 1, total_tokens < batch, max_seqlen outside 1..P), SP_EHIP. */
enum { SP_BAD_ID = 1, SP_BAD_CU0 = 2, SP_BAD_ORDER = 4, SP_BAD_LENGTH = 8, SP_BAD_TOTAL = 16 };
int sp_check_inputs(const sp_model* model, const int32_t* token_ids, const int32_t* cu_seqlens, int32_t batch,
                    int32_t total_tokens, int32_t max_seqlen, void* scratch, void* hip_stream,
                    int32_t* problems_host);

/* Byte offsets, inside a workspace laid out for (total_tokens, batch), of the
 * intermediate activations a forward leaves behind; for tests and profiling.
 * Each activation tensor is [k_active][rows][width] with `rows` >= total_tokens
 * (token-tile padded) in the model's activation type (float or bf16), row-major.
 *   x    [rows][H]  hidden state entering the next layer (after the last layer of a
 *                   partial forward: the final states; a whole forward forms the
 *                   final states of the first-token rows only where it can)
 *   qkv  [rows][3H] query | key | value projections of the last layer run; in bf16
 *                   mode the value slice is not written: the values are kept
 *                   transposed for the attention kernel, in
 *   vt   [H][rows]  value projection, feature-major (bf16 mode only)
 *   att  [rows][H]  attention output of the last layer run
 *   x1   [rows][H]  state after the attention block's LayerNorm
 *   g    [rows][F]  GELU(FFN up-projection)
 *   z    float32 [K][batch][C] per-student classifier outputs before the sum
 * and, written only when the last layer ran on the first-token rows (see
 * sp_config.last_layer_all_tokens; `x` then still holds the last layer's input), per
 * student first_rows rows, row b = sequence b:
 *   first_q    [first_rows][H]  the last layer's queries of the first tokens
 *   first_att  [first_rows][H]  its attention output for the first tokens */
typedef struct {
    size_t x, qkv, vt, att, x1, g, z;
    int32_t rows;      /* padded token rows per student */
    int32_t act_bytes; /* 4 or 2 */
    size_t first_q, first_att;
    int32_t first_rows;
    /* SP_DTYPE_FP8 only (0 otherwise), written by calls of >= 2048 token rows: e4m3 codes of 16 * value, one byte
     * per element, [k_active][rows][width]: xq, x1q, attq copies of x, x1 and att (width H); gq is GELU(FFN
     * up-projection) (width F; such calls do not write `g`). */
    size_t xq, x1q, gq, attq;
} sp_ws_layout;
int sp_workspace_layout(const sp_config* cfg, int32_t total_tokens, int32_t batch, sp_ws_layout* out);

/* Same as sp_forward but stops after `stop_after_layers` transformer layers
 * (0 = after the embedding LayerNorm) without computing logits; the
 * intermediates can then be read through sp_workspace_layout.  For tests. */
int sp_forward_partial(const sp_model* model, const int32_t* token_ids, const int32_t* cu_seqlens,
                       int32_t batch, int32_t total_tokens, int32_t max_seqlen, int32_t k_active,
                       int32_t stop_after_layers, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Phases of one forward, in the order of the encoder layer (Section 2.1: the serial depth
 * of attention layers is what the students shorten; each layer is these steps). */
enum {
    SP_PHASE_EMBED = 0,   /* embedding gather + LayerNorm */
    SP_PHASE_QKV,         /* query/key/value projection */
    SP_PHASE_ATTENTION,   /* softmax(q k^T / sqrt(d)) v inside each sequence */
    SP_PHASE_OPROJ,       /* attention output projection + residual */
    SP_PHASE_LAYERNORM,   /* both LayerNorms of every layer */
    SP_PHASE_FFN_UP,      /* feed-forward up-projection + GELU */
    SP_PHASE_FFN_DOWN,    /* feed-forward down-projection + residual */
    SP_PHASE_HEAD,        /* pooling, per-student head, cross-student sum */
    SP_PHASE_LAST_FIRST,  /* every kernel of a last layer that is computed for the first-token rows only
                           * (sp_config.last_layer_all_tokens == 0 and the call is large enough); the
                           * phases above then cover the other layers alone */
    SP_PHASE_COUNT
};

/* sp_forward with HIP events recorded on hip_stream after every kernel launch; waits for
 * the stream and adds each phase's device time, in milliseconds and summed over layers,
 * into phase_ms_host[SP_PHASE_COUNT] (host).  A measurement aid: it creates and destroys
 * events and synchronises, so it is not for latency-critical callers. */
int sp_forward_profiled(const sp_model* model, const int32_t* token_ids, const int32_t* cu_seqlens,
                        int32_t batch, int32_t total_tokens, int32_t max_seqlen, int32_t k_active,
                        void* workspace, size_t workspace_bytes, float* logits_out, void* hip_stream,
                        float* phase_ms_host);

/* y[i] = GELU(x[i]) exactly as the epilogue of the bf16 FFN up-projection evaluates it (exact erf form through a
 * fitted complementary error function, fp32 arithmetic), before the rounding to bf16; x_device, y_device: device
 * float32 [n], 1 <= n <= 2^31.  For the test that bounds its distance from the erf definition.
 * Errors: SP_EINVAL, SP_ESHAPE, SP_EHIP. */
int sp_probe_gelu(const float* x_device, float* y_device, int64_t n, void* hip_stream);

/* The same for the GELU of the fp8 FFN up-projection (SP_DTYPE_FP8), whose result is stored as an e4m3 code: the
 * erf form through a shorter fit, within 1e-4 of the definition (a thirtieth of the code's step where the function is
 * smallest); y[i] is the value before the scaling and the rounding to e4m3.  Same arguments and errors. */
int sp_probe_gelu_fp8(const float* x_device, float* y_device, int64_t n, void* hip_stream);

/* codes_host[i] = the OCP e4m3 code (sign, 4 exponent bits with bias 7, 3 mantissa bits; no infinities, largest
 * finite value 448) the weight loader of SP_DTYPE_FP8 gives x_host[i]: round to nearest even, saturating; NaN -> 0x7f.
 * Host arrays of n elements; runs on the host.  For the test that pins the loader's rounding.
 * Errors: SP_EINVAL, SP_ESHAPE (n < 0). */
int sp_probe_e4m3(const float* x_host, int64_t n, uint8_t* codes_host);

/* What the matrix cores of the current GPU sustain on bf16 operands with nothing else in the way: a loop of the
 * 32x32x16 bf16 matrix instruction on register operands (no memory traffic, sixteen accumulator blocks per wave, one
 * wave per SIMD, every compute unit busy), run for about `milliseconds` (1..2000) after an untimed stretch that lets
 * the clock settle.  operand_kind 0: every element 0 or 1; 1: uniform in (-1, 1) with full mantissas, which is what
 * weights and activations look like and what the package power limit prices; 2 and 3: the same two kinds of data
 * for the fp8 (e4m3) 32x32x64 instruction of the quantised students' projections.  *tflops_host receives the rate.
 * The projection kernels' fractions of the published peak are quoted next to this measured ceiling.  Creates and
 * destroys two events and blocks until the run has finished: a measurement aid.
 *   scratch_device  device, >= 4 bytes, 4-byte aligned (practically never written)
 * Errors: SP_EINVAL, SP_ESHAPE, SP_EHIP. */
int sp_probe_mfma_rate(int32_t operand_kind, int32_t milliseconds, void* scratch_device, void* hip_stream,
                       float* tflops_host);

#ifdef __cplusplus
}
#endif
#endif /* SP_H_ */
