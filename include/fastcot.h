/* fastcot.h -- C ABI of the MI355X (gfx950) FastCoT Jacobi-decoding library.
 *
 * The library runs the hot path of FastCoT (arXiv 2311.08263): one causal-decoder forward
 * over the committed KV cache plus a window of W tokens (Sec. 4.3, Eq. 4), per-row greedy
 * argmax (Eq. 1/2), verification of the approximate tokens (Eq. 5), acceptance of the verified
 * prefix, commit of its K/V and the shift of the window (Sec. 4.3 "Cache Update").
 *
 * Conventions
 *   - Every function returns 0 on success or a negative fastcot_status; fastcot_last_error()
 *     gives a text for the last failure of a context (or of a context-less call).
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are ordinary
 *     host memory owned by the caller.  The library never allocates or frees device memory; it
 *     owns only its host-side context (and a few pinned host words inside it).
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream).  All device work
 *     of a context is enqueued on the stream given to fastcot_init.
 *   - Host arrays are row-major int32 unless stated otherwise.
 *   - Window size W ("window" below) is the number of query rows per sequence per step: slot 0
 *     carries the newest exact token, slots 1..W-1 approximate tokens.  The paper's window size
 *     c counts only the extra tokens, so W = c + 1 and W = 1 is autoregressive decoding
 *     (Sec. 3.1, Fig. 2 caption).
 *   - Calls on one context must not overlap in time.
 */
#ifndef FASTCOT_H
#define FASTCOT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FASTCOT_OK = 0,
    FASTCOT_EINVAL = -1,    /* bad argument */
    FASTCOT_ESTATE = -2,    /* call order (e.g. step before prefill) */
    FASTCOT_ECAPACITY = -3, /* batch / sequence / buffer / workspace capacity exceeded */
    FASTCOT_EHIP = -4,      /* a HIP runtime call failed */
    FASTCOT_ENOMEM = -5     /* host allocation failed */
} fastcot_status;

enum { FASTCOT_F32 = 0, FASTCOT_BF16 = 1 };

/* Llama-style decoder shape plus capacities.  dtype is the storage type of the weights; the KV
 * cache is fp32 for fp32 models and bf16 planes for bf16 models (see FASTCOT_OPT_KV_PLANES);
 * activations, accumulation, softmax and norm statistics are always fp32. */
typedef struct fastcot_config {
    int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
    float rms_eps, rope_base;
    int32_t dtype;
    int32_t max_batch; /* sequences per step */
    int32_t max_seq;   /* KV-cache positions per sequence, also capacity of the token buffer */
    int32_t window;    /* W, query rows per sequence per step */
} fastcot_config;

/* Tensors of the model, in the caller's canonical layout: linear weights row-major [in][out]
 * (y = x . W), the embedding row-major [vocab][d_model], gains fp32 [d_model]. */
typedef enum {
    FASTCOT_T_EMB = 0, FASTCOT_T_WLM = 1, FASTCOT_T_GF = 2,
    FASTCOT_T_WQ = 3, FASTCOT_T_WK = 4, FASTCOT_T_WV = 5, FASTCOT_T_WO = 6,
    FASTCOT_T_WG = 7, FASTCOT_T_WU = 8, FASTCOT_T_WD = 9, FASTCOT_T_G1 = 10, FASTCOT_T_G2 = 11
} fastcot_tensor;

typedef struct fastcot_ctx fastcot_ctx;

/* Bytes of the library's packed device weight layout / of the device workspace (KV cache,
 * activations, token buffers, counters) for a configuration.  0 on an invalid configuration.
 * The activations are sized for the largest pass: a step of max_batch * window rows, or, for bf16 models
 * on the matrix-core kernels, a prompt chunk of up to 1024 rows in all (Sec. 4.1, the first forward). */
size_t fastcot_weight_bytes(const fastcot_config* cfg);
size_t fastcot_workspace_bytes(const fastcot_config* cfg);

/* Rearranges one tensor from the canonical layout into its place inside the packed weights.
 * d_canonical: device pointer, elements of cfg->dtype (gains: fp32); NULL for a gain tensor
 * means "all ones".  d_packed: device pointer to fastcot_weight_bytes() bytes.  `layer` is
 * ignored for EMB/WLM/GF.  Asynchronous on hip_stream; the canonical buffer may be reused once
 * the stream has passed this call.  Every tensor must be packed before fastcot_init's context
 * is used. */
int fastcot_pack_tensor(const fastcot_config* cfg, int32_t tensor, int32_t layer, const void* d_canonical,
                        void* d_packed, void* hip_stream);

/* The whole model in one call: d_canonical is one device buffer of fastcot_canonical_bytes() bytes holding every
 * tensor in the canonical layout above, tensor (t, layer) at byte offset fastcot_canonical_offset(cfg, t, layer)
 * (tensors follow each other in the order EMB, WLM, GF, then per layer WQ, WK, WV, WO, WG, WU, WD, G1, G2, each
 * start rounded up to 256 bytes; gains are fp32 and must be present: write ones for "no gain").  Equivalent to
 * fastcot_pack_tensor for every tensor; models too large to hold twice on the device are packed tensor by tensor
 * through a staging buffer instead.  (The library holds no weight generator: synthetic weights are inputs like
 * any others and come from the caller.)  fastcot_canonical_offset returns (size_t)-1 on bad arguments. */
size_t fastcot_canonical_bytes(const fastcot_config* cfg);
size_t fastcot_canonical_offset(const fastcot_config* cfg, int32_t tensor, int32_t layer);
int fastcot_pack_weights(const fastcot_config* cfg, const void* d_canonical, void* d_packed, void* hip_stream);

/* Creates a context over packed weights and a zero-initialised-or-not workspace (the library
 * initialises what it needs, synchronously).  Both device buffers must stay alive and untouched
 * by the caller until fastcot_free. */
int fastcot_init(const fastcot_config* cfg, const void* d_packed, void* d_workspace, size_t workspace_bytes,
                 void* hip_stream, fastcot_ctx** out);
void fastcot_free(fastcot_ctx* ctx);
const char* fastcot_last_error(const fastcot_ctx* ctx); /* ctx may be NULL */

/* Starts B sequences (Sec. 4.1: prompt construction is the caller's; Sec. 4.2: the buffer).
 * prompts: host [B][max_P], row b valid for lens[b] >= 1 tokens.  buffer_init: host [B][buf_len],
 * the initial Approximate Tokens Buffer, entry i being the first guess for generated token i;
 * buf_len <= max_seq.  Computes K/V of prompt tokens 0..len-2 and makes the last prompt token
 * slot 0 of the first window, so the first generated token comes from the first step.
 * Requires lens[b] - 1 + 2*window <= max_seq.  Synchronous. */
int fastcot_prefill(fastcot_ctx* ctx, int32_t B, const int32_t* prompts, int32_t max_P, const int32_t* lens,
                    const int32_t* buffer_init, int32_t buf_len);

/* One Jacobi step (Eq. 4, Eq. 5, cache update) for every unfinished sequence.  Host outputs,
 * each nullable: n_accepted[B] in 1..W (0 for a finished sequence); accepted[B][W], the first
 * n_accepted[b] entries valid; window_next[B][W], the next step's window (slot 0 exact).  With
 * all three NULL the call only enqueues work and returns without synchronising. */
int fastcot_jacobi_step(fastcot_ctx* ctx, int32_t* n_accepted, int32_t* accepted, int32_t* window_next);

/* Steps until every sequence has max_new_tokens exact tokens, or an exact token equals eos_id
 * (eos_id < 0: off; approximate EOS tokens are ignored), or max_steps steps were taken
 * (max_steps <= 0: no cap) -- the stop conditions of Sec. 4.4.  May be called after
 * fastcot_prefill, once.  Host outputs: out_ids[B][max_new_tokens]; out_len[B] (count of valid
 * ids, the EOS included); out_steps[B] (steps taken while the sequence was unfinished);
 * approx_tail[B][W-1] (nullable), the approximate tokens left in the window at stop.  Requires
 * buf_len >= max_new_tokens + 2*W and lens[b] - 1 + max_new_tokens + 2*W <= max_seq. */
int fastcot_generate(fastcot_ctx* ctx, int32_t max_new_tokens, int32_t max_steps, int32_t eos_id,
                     int32_t* out_ids, int32_t* out_len, int32_t* out_steps, int32_t* approx_tail);

/* Per-sequence state after the last completed call, host outputs, each nullable: n[B] committed
 * KV length; generated[B] exact tokens so far; done[B]; window[B][W] the window the next step
 * will feed; last_o[B][W] and last_K[B], the argmax rows and verified count of the last step.
 * Synchronises the stream. */
int fastcot_get_state(fastcot_ctx* ctx, int32_t* n, int32_t* generated, int32_t* done, int32_t* window,
                      int32_t* last_o, int32_t* last_K);

/* Changes the window size between two fastcot_jacobi_step calls (not during fastcot_generate): the next
 * step runs `window` rows per sequence, slot 0 the newest exact token, the rest from the buffer.  1 <= window
 * <= the rows a pass may have (the configured window, or 256 where the matrix-core path covers the model);
 * FASTCOT_ECAPACITY if a sequence has no room for it.  The accepted stream does not depend on the window
 * (Sec. 4.1); the step count does.  This is the hook an adaptive-window controller needs (Limitations). */
int fastcot_set_window(fastcot_ctx* ctx, int32_t window);

/* Per-sequence window sizes (ragged batches, Sec. 5.4 Time Composition; the window enters Eq. 4 and Eq. 5 per sequence):
 * windows: host, one entry per sequence of the last fastcot_prefill, 1 <= windows[b] <= the current batch
 * window W.  From the next step on sequence b verifies (Eq. 5), accepts and writes back to its buffer only the
 * first windows[b] rows of its W; its accepted stream, step count and approximate tokens are those of a run with
 * that window alone.  On the matrix-core path the step then computes only those rows, packed one sequence after
 * the other (FASTCOT_OPT_PACKED_ROWS, default 1; the rows of fastcot_debug_logits follow that order); the plain
 * kernels still compute W rows for every sequence.  Call after fastcot_prefill (which
 * resets every sequence to the batch window) and before fastcot_generate, or between fastcot_jacobi_step
 * calls; fastcot_generate's approx_tail and fastcot_answer's glimpse then hold windows[b] - 1 valid entries for
 * sequence b.  FASTCOT_ESTATE otherwise. */
int fastcot_set_windows(fastcot_ctx* ctx, const int32_t* windows);

/* Row layout of the next step (the rows of fastcot_debug_logits): row_start: host, B + 1 entries; the rows of
 * sequence b are row_start[b] .. row_start[b + 1] - 1, slot j of the sequence at row_start[b] + j, and
 * row_start[B] is the number of rows the step computes.  Dense (b * W) unless per-sequence windows packed the
 * rows (fastcot_set_windows).  Synchronises the stream when the layout has to be rebuilt.  Sec. 5.4 Time Composition. */
int fastcot_step_rows(fastcot_ctx* ctx, int32_t* row_start);

/* Ragged batches (Sec. 5.4 Time Composition, Table 2: a padded batch otherwise runs until its longest member ends): between
 * two fastcot_jacobi_step calls (not with fastcot_generate) a new sequence takes over slot `slot`, 0 <= slot <
 * the batch of the last fastcot_prefill.  prompt: host, len >= 1 token ids; buffer_init: host, buf_len ids
 * (the buf_len of that prefill).  The slot's former sequence is dropped; every other sequence keeps its state
 * and, Eq. 2 coupling no two sequences, its stream.  The newcomer's prompt is run through the model as a batch
 * of one (the sequence in slot 0 trades places with it meanwhile: two cache-to-cache copies of one sequence's
 * K/V).  Synchronises the stream.  FASTCOT_ESTATE before a prefill or after fastcot_generate; FASTCOT_EINVAL / FASTCOT_ECAPACITY as for fastcot_prefill. */
int fastcot_join(fastcot_ctx* ctx, int32_t slot, const int32_t* prompt, int32_t len, const int32_t* buffer_init);

/* Answer phase (Sec. 4.4 "Trigger Answer"), after fastcot_generate has returned: every sequence continues
 * from its prompt and exact tokens (already in the cache), the approximate tokens still in its window
 * (the glimpse; none for a sequence that ended with the EOS given to fastcot_generate), and the n_trigger
 * answer-trigger token ids (host, may be 0), and decodes greedily, one token per step, until
 * max_new_tokens or eos_id (< 0: off).  out_ids host
 * [B][max_new_tokens] (-1 past out_len[b]).  Afterwards the context needs a new fastcot_prefill. */
int fastcot_answer(fastcot_ctx* ctx, const int32_t* trigger_ids, int32_t n_trigger, int32_t max_new_tokens,
                   int32_t eos_id, int32_t* out_ids, int32_t* out_len);

/* Debug: if d_logits (device, fp32 [max_batch*W][vocab]) is non-NULL every following step also
 * stores the full logits there (row b*W + j); NULL switches it off. */
int fastcot_debug_logits(fastcot_ctx* ctx, float* d_logits);

/* Options of a context.
 * FASTCOT_OPT_PLAIN_KERNELS = 1 routes every step through the plain one-thread-per-output kernels (always used
 * for fp32 models, and for bf16 models whose shape the matrix-core kernels do not cover: head_dim other than 128,
 * or d_model / d_ffn / n_heads*head_dim not multiples of 256 -- fastcot_last_error() says so after fastcot_init);
 * 0 (default) uses the matrix-core kernels for bf16.
 * FASTCOT_OPT_GRAPH = 1 (default) replays a captured HIP graph per step; 0 launches kernels one by one.  A
 * context on the default (NULL) stream always launches one by one, since that stream cannot be captured.
 * FASTCOT_OPT_KV_PLANES (bf16 models): 2 (default) keeps every cached K/V value as a bf16 hi + bf16 lo pair
 * (4 bytes, ~16 mantissa bits); 1 keeps the hi plane only (2 bytes, plain bf16); 3 keeps the hi plane and one
 * byte of residual (3 bytes: the upper 24 bits of the fp32 value, which the attention kernel expands in
 * registers; faster than the pair only for steps of at most 16 rows per sequence over long contexts without
 * grouped-query heads).  Changing it invalidates the sequences: call fastcot_prefill again.
 * FASTCOT_OPT_COMPACT = 1 (default): whenever fastcot_generate finds finished sequences at one of its checks,
 * they trade slots (state and K/V cache) with unfinished ones so that the following steps run only the
 * unfinished sequences' rows; the order is restored before it returns.  0: finished sequences keep their rows.
 * FASTCOT_OPT_AUTOTUNE = 1 (default): at the first fastcot_prefill of a step shape with at most 32 rows, the
 * column-owner GEMMs that walk K in plain order (QKV, O) are timed on the model's own matrices with one / two
 * weight batches in flight or the whole K slice requested up front, and the fastest is kept.  The choice moves
 * loads, not additions: logits are the same bits whichever wins, in every process.  Everything that fixes the
 * order of the fp32 additions (K slices per owner, batch order) is chosen from the model shape alone.  Setting
 * any FASTCOT_PLAN_* value turns the measurement off: explicit choices win.
 * FASTCOT_OPT_KV_EMULATE (bf16 models, matrix-core kernels; a precision study, not a storage mode): value =
 * K mode + 16 * V mode; before a K (V) value is cached it is rounded as a narrower storage format would round it
 * (mode 0 as computed, 1 bf16, 2 fp16, 3 the upper 24 bits of fp32) and then kept in the two planes as usual, so
 * the logits show what that format would cost before a kernel for it exists.  Needs a new fastcot_prefill.
 * FASTCOT_OPT_ACT_EMULATE (bf16 models, steps of at most 32 rows; a precision study): a mask over the five GEMMs
 * (bit 0 QKV, 1 O, 2 gate/up, 3 down, 4 LM head); a GEMM whose bit is set takes its input activations as plain
 * bf16 instead of the bf16 hi + lo pair the kernels use.
 * FASTCOT_OPT_DEBUG_STAGES: run only the first `value` stages of a forward (per layer: QKV, attention, O,
 * gate/up, down); negative (default) = all. */
enum { FASTCOT_OPT_PLAIN_KERNELS = 1, FASTCOT_OPT_GRAPH = 2, FASTCOT_OPT_KV_PLANES = 3, FASTCOT_OPT_COMPACT = 4,
       FASTCOT_OPT_AUTOTUNE = 5, FASTCOT_OPT_DEBUG_STAGES = 6, FASTCOT_OPT_KV_EMULATE = 7, FASTCOT_OPT_ACT_EMULATE = 8,
       FASTCOT_OPT_PACKED_ROWS = 9 };

/* Launch-plan values, also set through fastcot_set_option.  They are measurement aids: defaults are chosen from
 * the model shape, and which values exist may change with the kernels.  The five GEMMs are numbered QKV, O,
 * gate/up, down, LM head.
 * FASTCOT_PLAN_NW + g: workgroups of GEMM g (each owns at most 8 tiles of 16 columns over all of K).
 * FASTCOT_PLAN_KS + g (g < 4): workgroups per column owner, each taking 1/value of K (1..8); their partial tiles
 * meet through memory and the last to arrive adds them in slice order.  The workgroup count must be a multiple.
 * FASTCOT_PLAN_SB + g: weight batches in flight per wave: 0 two, 1 one, 2 the wave's whole K slice up front.
 * FASTCOT_PLAN_ROT + g: 1 = every wave walks its K batches in an order rotated by workgroup and wave.
 * FASTCOT_PLAN_CO_SINGLE: 0 / 1 = two / one batch in flight for every GEMM, 2 (default) = per GEMM (PLAN_SB).
 * FASTCOT_PLAN_ATTN_SPLITS: key-range splits the attention launch provides (1..16).
 * FASTCOT_PLAN_ATTN_BLOCKS: key blocks of 32 positions per attention workgroup: of the launched splits,
 * ceil(blocks / value) work on a sequence, the rest exit.
 * FASTCOT_PLAN_ATTN_MANY_ROWS: which passes use the attention kernel for many rows per sequence (workgroups of
 * 128 rows that walk the keys once; prompt chunks): 0 none, 1 (default) passes of at least 64 rows per sequence
 * whose launch gives at least half of the compute units a workgroup, 2 every pass of more than 32 rows. */
enum { FASTCOT_PLAN_NW = 100, FASTCOT_PLAN_KS = 105, FASTCOT_PLAN_SB = 110, FASTCOT_PLAN_ROT = 115,
       FASTCOT_PLAN_CO_SINGLE = 120, FASTCOT_PLAN_ATTN_SPLITS = 121, FASTCOT_PLAN_ATTN_BLOCKS = 122,
       FASTCOT_PLAN_ATTN_MANY_ROWS = 123 };
int fastcot_set_option(fastcot_ctx* ctx, int32_t option, int32_t value);

/* Debug: copies `count` floats of an activation buffer of the last forward to the host after
 * synchronising: what = 0 residual stream [rows][d_model], 1 rotated queries (MFMA path: [rows][H*Dh]),
 * 2 attention output [rows][H*Dh], 3 MLP hidden [rows][d_ffn]. */
int fastcot_debug_read(fastcot_ctx* ctx, int32_t what, float* host, size_t count);

/* Wall time of the steps of the last fastcot_generate, measured with HIP events on the
 * context's stream: ms[i] for step i, up to cap entries; *n_steps = steps taken. */
int fastcot_step_times(fastcot_ctx* ctx, float* ms, int32_t cap, int32_t* n_steps);

/* Runs `iters` forward passes of the current state (no accept, state unchanged), launching
 * kernels one by one with a HIP event pair around each, and reports per kernel kind the mean
 * duration of one launch in ms and the launches per step.  kinds: see fastcot_kernel_name(); kind
 * "empty_kernel" is the same event pair around a kernel that does nothing (what the pair itself adds).
 * Host outputs sized FASTCOT_N_KERNEL_KINDS. */
enum { FASTCOT_N_KERNEL_KINDS = 16 };
int fastcot_profile_step(fastcot_ctx* ctx, int32_t iters, float* mean_ms, int32_t* launches_per_step);
const char* fastcot_kernel_name(int32_t kind);

/* Kernel-isolation entry points (the same kernels the step uses, on raw device pointers).
 *
 * Window-causal attention (Eq. 2 conditioning as a mask): q device fp32 [W][H][Dh] (already
 * rotated); k_cache / vt_cache in the library's single-plane cache layout for one sequence: per kv head
 * max_seq/32 blocks of 32 positions x Dh elements, each block stored in the order of the attention
 * kernel's matrix-core operand fragments (written by fastcot_kv_scatter; max_seq and Dh multiples of 32),
 * elements of `dtype`, positions 0..n+W-1 filled; row j attends positions 0..n+j.  out device fp32 [W][H*Dh].  scratch: device,
 * fastcot_attn_scratch_bytes() bytes, zeroed once by the caller before first use.
 * fastcot_kv_scatter writes canonical k, v (device, [S][Hkv][Dh], `dtype`) into that layout. */
size_t fastcot_attn_scratch_bytes(int32_t W, int32_t H, int32_t Dh);
int fastcot_kv_scatter(const void* d_k, const void* d_v, int32_t S, int32_t Hkv, int32_t Dh, int32_t max_seq,
                       int32_t dtype, void* d_k_cache, void* d_vt_cache, void* hip_stream);
int fastcot_attn_window(const float* d_q, const void* d_k_cache, const void* d_vt_cache, int32_t n, int32_t W,
                        int32_t H, int32_t Hkv, int32_t Dh, int32_t max_seq, int32_t dtype, float* d_out,
                        void* d_scratch, void* hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): fastcot_attn_window with the kernel's scratch (split-key partial results and arrival
 * counters) in an array built into the library instead of a caller buffer.  Arguments and results as for
 * fastcot_attn_window.  Limits: H <= 64 query heads and W <= 16 window rows (FASTCOT_ECAPACITY beyond, with a
 * text in fastcot_last_error(NULL)); the array is about 8.5 MiB per GPU the library runs on, held until the
 * process ends.  The call allocates nothing and frees nothing.  All calls on one GPU share that GPU's array:
 * calls that overlap in time on one GPU (different streams or threads) race and give undefined results. */
int fastcot_attn_window_noalloc(const float* d_q, const void* d_k_cache, const void* d_vt_cache, int32_t n, int32_t W,
                                int32_t H, int32_t Hkv, int32_t Dh, int32_t max_seq, int32_t dtype, float* d_out,
                                void* hip_stream);

/* Measurement aids.  fastcot_stream_read: one plain streaming read of `bytes` (multiple of 16) device bytes at
 * d_src (16-byte aligned), shaped like the weight stream of the step's GEMMs (one workgroup per compute unit,
 * contiguous kilobytes per wave, 16 loads in flight); d_sink16 is a 16-byte device scratch the kernel may
 * write.  Timed by the caller, it gives the read bandwidth the device delivers to the simplest kernel: a
 * second denominator beside the published HBM peak.  fastcot_stream_read_chain: n_launches such launches back
 * to back, launch i reading launch_bytes[i] (host array; rounded down to whole kilobytes, each at most
 * src_bytes) from consecutive parts of the src_bytes at d_src (wrapping around): with the byte counts of a
 * step's kernels this is what the step would cost if every kernel only read its weights -- the floor of a
 * step made of separate launches. */
int fastcot_stream_read(const void* d_src, size_t bytes, void* d_sink16, void* hip_stream);
int fastcot_stream_read_chain(const void* d_src, size_t src_bytes, const uint64_t* launch_bytes, int32_t n_launches,
                              void* d_sink16, void* hip_stream);

/* LM head fused with argmax (Eq. 1/2, lowest id on ties): act device fp32 [M][d] (already
 * normalised), packed W_lm as written by fastcot_lmhead_pack from canonical bf16 [d][V];
 * ids device int32 [M], top device fp32 [M] (the winning logit); d_top2 nullable fp32 [M], the largest logit
 * among all other ids (top - top2 is the margin of the decision; asking for it makes the call write the
 * logits, to d_logits or to the scratch); d_logits nullable fp32 [M][V].
 * scratch: device, fastcot_lmhead_scratch_bytes() bytes, zeroed once by the caller. */
size_t fastcot_lmhead_packed_bytes(int32_t d, int32_t V);
size_t fastcot_lmhead_scratch_bytes(int32_t M, int32_t d, int32_t V);
int fastcot_lmhead_pack(const void* d_canonical_bf16, int32_t d, int32_t V, void* d_packed, void* hip_stream);
int fastcot_lmhead_argmax(const float* d_act, const void* d_packed, int32_t M, int32_t d, int32_t V,
                          int32_t* d_ids, float* d_top, float* d_top2, float* d_logits, void* d_scratch, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* FASTCOT_H */
