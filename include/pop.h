/*
 * pop.h -- C ABI of the POP (Prefill-Only Pruning) prefill library for AMD MI355X (gfx950).
 *
 * The library computes the pruned prefill forward pass of a decoder-only transformer as defined in
 * the POP paper, Sec. 3.3 ("Prefill-Only Pruning for Efficient Inference"):
 *   - layers 1..L_keep run in full for the prompt body (Sec. 2.1, layer forward + K/V generation +
 *     cache append);
 *   - layers L_keep+1..L are skipped for the body (identity on the hidden state) but still receive
 *     their KV-cache entries through the "independent KV projections"
 *         k_l = RoPE(LN(x_l) W_l^K),  v_l = LN(x_l) W_l^V
 *     with the layer's own norm scale and projection matrices;
 *   - the last prompt token of every sequence (the boundary token) is processed at full depth as the
 *     first decode step ("Boundary Handling for the Last Input Token"), so the first generated
 *     token's logits come from the whole model.
 * The decode operator of Sec. 3.2 (one token through all layers against the cache) is exported as
 * pop_decode_step; it is the same code the boundary token runs.
 *
 * Conventions
 *   Memory     Every DEVICE pointer is caller-owned device memory (weights, cache pool, workspace,
 *              logits).  The library allocates no device memory: only small host structs and, per
 *              cache, two pinned host buffers of the size of a call's int32 metadata (the calls copy
 *              that to the device from there), released by the matching pop_free_model /
 *              pop_cache_destroy.  HOST pointers are read during the call only.
 *   Layout     All matrices are row-major [out_features, in_features] (the contraction index is
 *              contiguous), elements bf16.  Norm scales are fp32 [d_model].
 *   Precision  POP_DTYPE_BF16 is the production path (bf16 weights and cache, fp32 accumulation
 *              and residual stream, MFMA kernels).  POP_DTYPE_F32 runs every step in fp32 with fp32
 *              weights, embedding rows and cache entries (wherever this header says bf16, read
 *              fp32); it is a slow checking path for small models: sequences of at most 15000
 *              tokens (POP_EUNSUPPORTED beyond).
 *   Errors     Every call returns a pop_status.  Argument errors are detected on the host before
 *              anything is enqueued and leave cache contents and lengths unchanged;
 *              pop_last_error() then returns a message (thread-local, static storage).
 *   Asynchrony On POP_OK the work is enqueued on `stream` (a hipStream_t); outputs are valid once
 *              the caller has synchronised with it.  Host input arrays may be reused on return.
 *   Determinism Same inputs give bit-identical outputs (no floating-point atomics).
 *   Alignment  Device pointers must be 16-byte aligned (256 for the workspace).
 */
#ifndef POP_H_
#define POP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pop_model pop_model; /* opaque host-side handle over caller-owned device weights */
typedef struct pop_cache pop_cache; /* opaque host-side handle over a caller-owned device pool   */
typedef void* pop_stream;           /* a hipStream_t (0 = the null stream)                        */

typedef enum {
  POP_OK = 0,
  POP_EINVAL = -1,       /* NULL pointer, bad count, bad l_keep, token id out of range, ...        */
  POP_ESHAPE = -2,       /* model shape the kernels do not cover                                   */
  POP_EALIGN = -3,       /* misaligned device pointer                                              */
  POP_ENOSPACE = -4,     /* not enough pages, page-table columns, workspace or pool bytes          */
  POP_ESTATE = -5,       /* e.g. decode on a sequence that was never prefilled                     */
  POP_EHIP = -6,         /* a HIP runtime call or launch failed                                    */
  POP_EUNSUPPORTED = -7  /* valid request the build does not implement (e.g. fp32 beyond 15000 tokens)*/
} pop_status;

/* Message of the last failing call on this thread ("" if none).  Never freed by the caller. */
const char* pop_last_error(void);
/* Library version string. */
const char* pop_version(void);

enum { POP_DTYPE_F32 = 0, POP_DTYPE_BF16 = 1 };
enum { POP_ACT_SILU = 0, POP_ACT_GELU_TANH = 1 };

/* Model shape (Sec. 2.1: L layers, hidden size d, GQA attention block + gated FFN block). */
typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  int32_t dtype;           /* POP_DTYPE_* (see Precision above)                                    */
  int32_t act;             /* POP_ACT_*: FFN = (act(m Wg^T) * (m Wu^T)) Wd^T                       */
  float rms_eps;           /* LN(x) = x * rsqrt(mean(x^2) + rms_eps) * gamma                       */
  float rope_theta;        /* RoPE base of global-attention layers                                 */
  float rope_theta_local;  /* RoPE base of sliding-window layers                                   */
  int32_t sliding_window;  /* 0 = none; W > 0: a local layer's row t sees positions t-W+1 .. t     */
  int32_t global_every;    /* 0 = every layer global; g > 0: 1-based layer l is global iff l%g==0  */
  int32_t page_size;       /* tokens per KV-cache page, a power of two (16)                        */
  /* Optional 8-bit KV cache (a family extra, not part of the method; all zero = bf16 entries).           */
  int32_t kv_dtype;        /* POP_KV_BF16 or POP_KV_FP8_E4M3                                       */
  float k_scale, v_scale;  /* POP_KV_FP8_E4M3: an entry x is stored as the e4m3 code of x / scale and
                              read back as code value * scale; finite and > 0 (ignored for bf16)    */
} pop_config;
/* POP_KV_FP8_E4M3: the cache append of Sec. 2.1 stores every K/V element as the nearest value of the 8-bit
 * floating-point format with 4 exponent bits (bias 7), 3 mantissa bits and no infinities (largest finite value
 * 448), ties to the even mantissa, magnitudes beyond 448 clamped to 448; keys are rotated first.  Attention runs
 * on the updated cache (Sec. 2.1): EVERY attention, in the prefill as in decode steps, reads the stored entries,
 * a token's own entry included, so the boundary token's pass through the kept layers inside the prefill stays
 * identical to its decode step.  With POP_DTYPE_F32 the cache keeps fp32 entries that hold the rounded values. */
enum { POP_KV_BF16 = 0, POP_KV_FP8_E4M3 = 1 };

typedef struct {
  const void* norm_in;   /* DEVICE fp32 [d]                 input norm scale (the LN of Sec. 2.1)  */
  const void* wqkv;      /* DEVICE bf16 [Dq + 2 Dkv, d]     rows ordered W^Q | W^K | W^V           */
  const void* wo;        /* DEVICE bf16 [d, Dq]                                                    */
  const void* norm_post; /* DEVICE fp32 [d]                 norm in front of the FFN block         */
  const void* w_gate_up; /* DEVICE bf16 [2 f, d]            rows ordered gate | up                 */
  const void* w_down;    /* DEVICE bf16 [d, f]                                                     */
  /* Optional per-head QK-norm (a family extra, not part of the method; both NULL = off, both or
     neither): every query head is RMS-normalised over head_dim with scale q_norm, every key head with
     k_norm (same rms_eps), before RoPE; in kept layers, in the pruned layers' key projection and in
     decode steps alike. */
  const void* q_norm;    /* DEVICE fp32 [head_dim] or NULL                                         */
  const void* k_norm;    /* DEVICE fp32 [head_dim] or NULL                                         */
} pop_layer_weights;

typedef struct {
  const void* embed;               /* DEVICE bf16 [vocab, d]                                       */
  const void* final_norm;          /* DEVICE fp32 [d]                                              */
  const void* lm_head;             /* DEVICE bf16 [vocab, d]                                       */
  const pop_layer_weights* layers; /* HOST array of n_layers entries (copied by pop_load_weights)  */
} pop_weights;

/*
 * Validates the shape and records the weight pointers (borrowed: they must outlive the model).
 * Host-only, enqueues nothing, allocates no device memory.
 * Errors: POP_EINVAL (NULL, non-positive sizes, Hq % Hkv != 0, unknown kv_dtype, bad k_scale / v_scale),
 * POP_ESHAPE (head_dim not in
 * {64,128,256}, d_model or d_ffn not a multiple of 8, page_size not a power of two in 1..256, a bf16
 * weight matrix of 2 GiB or more), POP_EALIGN; POP_EINVAL also if a layer has only one of q_norm / k_norm.
 */
pop_status pop_load_weights(const pop_config* cfg, const pop_weights* w, pop_model** out);
void pop_free_model(pop_model* m);

/*
 * KV cache (Sec. 2.1, cache append) stored in pages.  Device layout, bf16 (one byte per element, the e4m3 code,
 * with POP_KV_FP8_E4M3):
 *     pool[layer][kv][page][kv_head][slot_in_page][head_dim],   kv = 0 for K, 1 for V.
 * Entry t of sequence b lives in page block_table[b][t / P] at offset t % P.
 */
size_t pop_cache_bytes(const pop_config* cfg, int32_t n_pages);
/* Upper bound of the workspace pop_prefill / pop_decode_step need for at most max_tokens packed
 * tokens in at most max_seqs sequences whose page tables have max_pages_per_seq columns. */
size_t pop_workspace_bytes(const pop_config* cfg, int32_t max_tokens, int32_t max_seqs,
                           int32_t max_pages_per_seq);
/* Wraps a device pool of at least pop_cache_bytes(cfg, n_pages) bytes.  Contents are not touched.
 * Errors: POP_EINVAL, POP_EALIGN, POP_ENOSPACE (bytes too small). */
pop_status pop_cache_create(const pop_config* cfg, void* dev_pool, size_t bytes, int32_t n_pages,
                            int32_t max_seqs, int32_t max_pages_per_seq, pop_cache** out);
void pop_cache_destroy(pop_cache* c); /* does not free dev_pool */
/* Number of live sequences and their current lengths (host_out has room for max_seqs values). */
int32_t pop_cache_n_seqs(const pop_cache* c);
pop_status pop_cache_seq_lens(const pop_cache* c, int32_t* host_out);
/* The page table the cache object holds (Sec. 2.1, cache append: where the entries of each sequence are) and the
 * current lengths: host_out HOST [max_seqs][max_pages_per_seq] receives the page ids the last pop_prefill was
 * given (negative = unassigned; all negative before the first prefill), host_seq_lens HOST [max_seqs] (may be
 * NULL) the lengths as of now.  Read-only: the table stays the caller's to decide (see pop_prefill_args), this
 * call hands back the copy the library addresses the pool with.  POP_EINVAL on NULL. */
pop_status pop_cache_block_table(const pop_cache* c, int32_t* host_out, int32_t* host_seq_lens);

/*
 * Cache slot of every packed token (integer, host-only):
 *     slot[cu_seqlens[b] + t] = block_table[b * max_pages_per_seq + t / P] * P + t % P.
 * This is the function pop_prefill uses for its own addressing.
 * Errors: POP_EINVAL (NULL, n_seqs < 1, cu_seqlens not starting at 0 / not strictly increasing,
 * page id outside [0, n_pages), a page used twice), POP_ENOSPACE (a sequence needs more columns
 * than max_pages_per_seq or reaches an unassigned (negative) entry).
 */
pop_status pop_slot_map(const int32_t* host_cu_seqlens, int32_t n_seqs, const int32_t* host_block_table,
                        int32_t max_pages_per_seq, int32_t page_size, int32_t n_pages,
                        int32_t* host_slots_out);

typedef struct {
  const int32_t* tokens;       /* HOST [T] packed token ids of all sequences                        */
  const int32_t* cu_seqlens;   /* HOST [n_seqs + 1], cu[0] = 0, strictly increasing, cu[n_seqs] = T */
  int32_t n_seqs;
  const int32_t* block_table;  /* HOST [n_seqs][max_pages_per_seq] page ids, negative = unassigned;
                                  must cover every position the sequences will reach, including
                                  later decode steps.  The table is the CALLER's: which page a sequence
                                  gets is the serving engine's allocation policy (free lists, prefix
                                  sharing, eviction), not part of the method, so the library exports no
                                  allocator; it validates the table it is given (pop_slot_map's rules),
                                  copies it into the cache object, and reports that copy and the lengths it
                                  has recorded through pop_cache_block_table / pop_cache_seq_lens       */
  const void* embeds;          /* DEVICE bf16 [sum of counts, d] or NULL: rows that replace the
                                  embedding lookup (e.g. visual tokens fed as hidden states)        */
  const int32_t* embed_ranges; /* HOST [n_ranges][3] = (seq, first_pos, count), rows of `embeds`
                                  consumed in this order; ranges must not overlap                   */
  int32_t n_ranges;
  int32_t l_keep;              /* 0 .. n_layers: layers 1..l_keep are kept for the body, the deep
                                  block l_keep+1..L is pruned (ignored when skip_layers is given)   */
  int32_t mode;                /* POP_MODE_POP: the last token of each sequence is the boundary token:
                                  full depth, logits returned.
                                  POP_MODE_BODY_ONLY: every given token is a body token (pruned in
                                  the pruned layers); no logits.  pop_decode_step on the next token
                                  then completes the same computation.
                                  POP_MODE_NO_BOUNDARY (ablation, Sec. 4.4): every given token is a
                                  body token and the logits are the final norm and LM head of the
                                  pruned model's output for each sequence's last token.             */
  /* The fields below may be left zero: zero means the method as published. */
  const int32_t* skip_layers;  /* HOST [n_skip] or NULL.  A general skip set (Sec. 2.2), applied to
                                  the body tokens of the prefill only: 1-based layer indices,
                                  strictly increasing.  A pruned layer passes its input on unchanged
                                  and stores the K/V projections of that input (Sec. 3.3), so pruned
                                  layers separated by a kept layer project different hidden states.
                                  NULL: the deep block given by l_keep.  Non-NULL with n_skip = 0:
                                  nothing is pruned.                                                */
  int32_t n_skip;
  int32_t no_kv_projection;    /* 1 (ablation, Sec. 4.4): pruned layers store nothing for body
                                  tokens; the boundary token and every later token then see, in
                                  those layers, only the entries from the first full-depth token on
                                  (positions stay absolute).  0: independent KV projections.        */
  int32_t window_kv_writes;    /* 1: a pruned sliding-window layer stores only the body entries that the
                                  first full-depth token (position len-1 in POP_MODE_POP, len
                                  otherwise) can still see, i.e. positions > that position - W; later
                                  tokens see even less of the body, so no result changes and the
                                  K/V-only projection of such a layer shrinks to at most W rows per
                                  sequence.  The other slots keep what they held.  0: all entries.   */
  const float* gates;          /* HOST [n_layers] or NULL.  Prefill-stage virtual gates (Sec. 3.1 in the
                                  stage-aware form of Sec. 3.2; the paper's tool for measuring layer
                                  importance, not part of serving): a layer that runs in full multiplies
                                  both of its residual branches, the attention output and the FFN
                                  output, by gates[l-1]; its K/V entries do not depend on its own gate.
                                  NULL: all 1.  Only with POP_MODE_BODY_ONLY or POP_MODE_NO_BOUNDARY,
                                  where every given token is a prefill-stage token; the decode-stage
                                  gates of the last prompt token and of later tokens go to
                                  pop_decode_step_gated.                                              */
} pop_prefill_args;
enum { POP_MODE_POP = 0, POP_MODE_BODY_ONLY = 1, POP_MODE_NO_BOUNDARY = 2 };

/*
 * Pruned prefill (Sec. 3.3).  Starts sequences 0..n_seqs-1 from empty (a cache that was in use is
 * reset), writes the K/V entries of all n_layers layers for every given token and, in POP mode, the
 * boundary tokens' next-token logits.
 *   dev_logits   DEVICE fp32 [n_seqs, vocab]; may be NULL in POP_MODE_BODY_ONLY.
 * With no_kv_projection the cache pages of a pruned layer keep whatever they held at the body
 * positions; the cache object remembers that those entries do not exist, and pop_decode_step /
 * pop_generate honour it until the next pop_prefill.
 *   dev_workspace DEVICE scratch of at least pop_workspace_bytes(cfg, T, n_seqs, max_pages_per_seq).
 * Errors (all before any launch): POP_EINVAL (NULL, l_keep outside [0, L], skip_layers not strictly
 * increasing or outside [1, L], n_skip without skip_layers, unknown mode or switch value, gates in
 * POP_MODE_POP or a gate that is not finite, n_seqs < 1
 * or above the cache's max_seqs, an empty sequence, token id outside [0, vocab), bad embed range),
 * POP_ENOSPACE
 * (pages, workspace), POP_EALIGN.  POP_EHIP if a launch fails.
 */
pop_status pop_prefill(pop_model* m, pop_cache* c, const pop_prefill_args* args, float* dev_logits,
                       void* dev_workspace, size_t workspace_bytes, pop_stream stream);

/*
 * One decode step (Sec. 3.2): token host_tokens[b] is appended to sequence b at position len_b, runs
 * all n_layers layers against the cache, and its next-token logits are written to
 * dev_logits[b, :] (DEVICE fp32 [n_seqs, vocab]).  n_seqs must equal the cache's live sequences.
 * Errors: POP_EINVAL, POP_ESTATE (no prefilled sequences), POP_ENOSPACE (a sequence has no page
 * assigned for position len_b, or workspace too small), POP_EHIP.
 */
pop_status pop_decode_step(pop_model* m, pop_cache* c, const int32_t* host_tokens, int32_t n_seqs,
                           float* dev_logits, void* dev_workspace, size_t workspace_bytes,
                           pop_stream stream);
/* The same step with decode-stage virtual gates (Sec. 3.1 / 3.2, see pop_prefill_args.gates): layer l
 * multiplies both of its residual branches by host_gates[l-1] (HOST [n_layers]; NULL = all 1, which is
 * pop_decode_step).  POP_EINVAL also if a gate is not finite. */
pop_status pop_decode_step_gated(pop_model* m, pop_cache* c, const int32_t* host_tokens, int32_t n_seqs,
                                 const float* host_gates, float* dev_logits, void* dev_workspace,
                                 size_t workspace_bytes, pop_stream stream);

/*
 * Greedy generation (Sec. 3.2: prefill, then the decode loop with the full model): pop_prefill in
 * POP_MODE_POP (or POP_MODE_NO_BOUNDARY), then max_new_tokens tokens per sequence.  Token 0 is the index of the largest
 * boundary-token logit (lowest index on ties); token s > 0 is chosen the same way from the logits
 * of a decode step on token s-1.  Once a sequence has produced eos_token (>= 0; pass -1 for none)
 * all its later tokens are eos_token (its steps are still computed, so all sequences stay in
 * step).  Everything is enqueued without a host synchronisation: tokens are chosen and fed back on
 * the device.
 *   dev_tokens_out DEVICE int32 [n_seqs, max_new_tokens]
 *   dev_logits     DEVICE fp32 [n_seqs, vocab]: scratch for every step; holds the last step's logits
 *   dev_workspace  at least pop_generate_workspace_bytes(cfg, T, n_seqs, max_pages_per_seq, max_new_tokens)
 * The block table must assign pages for positions up to len_b + max_new_tokens - 2.  Afterwards the
 * cache holds len_b + max_new_tokens - 1 entries per sequence (the last chosen token is not fed).
 * Errors as pop_prefill, plus POP_EINVAL (max_new_tokens < 1, POP_MODE_BODY_ONLY, gates given,
 * eos_token >= vocab) and POP_ENOSPACE (pages for the generated tokens, workspace); all before any launch.
 */
size_t pop_generate_workspace_bytes(const pop_config* cfg, int32_t max_tokens, int32_t max_seqs,
                                    int32_t max_pages_per_seq, int32_t max_new_tokens);
pop_status pop_generate(pop_model* m, pop_cache* c, const pop_prefill_args* args, int32_t max_new_tokens,
                        int32_t eos_token, int32_t* dev_tokens_out, float* dev_logits, void* dev_workspace,
                        size_t workspace_bytes, pop_stream stream);

/*
 * Optional per-step timing for benchmarks.  While enabled, pop_prefill brackets every launch of the
 * steps below with HIP events on the caller's stream (this adds a little launch overhead, so whole-
 * call latency should be measured with timing disabled).  pop_timing_read waits for the recorded
 * events, adds the elapsed time and launch count of each step kind since the last read into
 * ms_out[POP_N_STEPS] / launches_out[POP_N_STEPS] (HOST arrays) and clears the record.
 * Step kinds follow the layer forward of Sec. 2.1 and the pruned-layer / boundary split of Sec. 3.3.
 */
enum {
  POP_STEP_EMBED = 0,     /* embedding gather + RoPE tables                       */
  POP_STEP_NORM = 1,      /* RMSNorm (both norms of a kept layer)                 */
  POP_STEP_QKV_GEMM = 2,
  POP_STEP_ROPE_WRITE = 3, /* RoPE + cache append (kept layers)                   */
  POP_STEP_ATTENTION = 4,
  POP_STEP_O_GEMM = 5,
  POP_STEP_GATE_UP_GEMM = 6,
  POP_STEP_DOWN_GEMM = 7,
  POP_STEP_KV_ONLY_NORM = 8,  /* pruned layers: shared-statistics norm            */
  POP_STEP_KV_ONLY_GEMM = 9,  /* pruned layers: batched K/V projection            */
  POP_STEP_KV_ONLY_WRITE = 10, /* pruned layers: RoPE + cache append              */
  POP_STEP_BOUNDARY = 11,     /* boundary rows: deep layers + final norm + LM head */
  POP_STEP_DOWN_ADD_NORM = 12, /* long prompts: adds the K parts of the down projection to the hidden state and
                                  writes the next layer's normalised input (or only adds, after the last kept layer) */
  POP_N_STEPS = 13
};
pop_status pop_timing_enable(pop_model* m, int32_t enable);
pop_status pop_timing_read(pop_model* m, float* ms_out, int32_t* launches_out);

#ifdef __cplusplus
}
#endif
#endif /* POP_H_ */
