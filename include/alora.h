/* libalora -- Activated LoRA (aLoRA) attention over a reused base-model KV cache,
 * hand-written HIP for AMD MI355X (gfx950).  Plain C ABI: pointers and sizes only.
 *
 * The operation (paper Section 2, Eq.6, with Eq.1-4 of its background section):
 * for every sequence b of a packed batch, tokens at absolute positions before the
 * invocation index k_b use the base projection weights; tokens at positions >= k_b use
 *      y = W_p x + s_a * B_{a,p} (A_{a,p} x),      p in {q, k, v},  a = adapter of b.
 * Keys and values of positions already in the cache are taken from it unchanged
 * (Proposition 1); only the new rows are projected, rotated (rotary embedding),
 * appended behind the cached rows, and the new queries attend causally -- each over cache
 * rows 0..its own position, itself included (Eq.4) -- with softmax scale 1/sqrt(head_dim)
 * (Eq.1) and grouped-query head sharing (kv head = q head / (n_q_heads/n_kv_heads)).
 *
 * Conventions
 *   - "HOST" pointers are ordinary host memory, read (and for seq_len written) during the
 *     call; "DEVICE" pointers are HIP device memory of the context's GPU.
 *   - All matrices are row-major.  W is stored [out, in], A [rank, in], B [out, rank].
 *   - dtype selects the storage type of x, W, A, B, gains, cache and outputs
 *     (ALORA_BF16 or ALORA_F32); accumulation is always fp32.
 *   - Rotary embedding: "rotate-half" pairing -- within a head, element c < head_dim/2 is
 *     paired with element c + head_dim/2 and the pair is rotated by pos * theta^(-2c/head_dim);
 *     absolute positions; applied to q and k before k is stored, never to v.
 *   - k_b is the 0-based absolute position of the first adapted token (the paper's
 *     1-based t_invoke minus 1).  k_b may lie before the cached length (the cache already
 *     holds adapted rows, as during decoding), inside the new rows, or beyond them (all new
 *     rows are base rows).  adapter -1 means base model only.  k_b = 0 with an empty cache
 *     is standard LoRA (Eq.5).
 *   - Calls are asynchronous on the given stream.  The library owns only its context
 *     (a workspace that grows on demand, staged copies of the small HOST arrays, a rotary
 *     table); it never frees or keeps caller memory.  One context per stream; a context
 *     is not thread-safe.  When a call needs a larger workspace or a longer rotary table than
 *     the context holds, the context synchronises the DEVICE, frees the old block and allocates
 *     a new one before it enqueues anything (the first call of a given size, typically); calls
 *     that fit are enqueued without any synchronisation or allocation.
 *   - Every argument is validated on the host before anything is launched.  On any error
 *     nothing has been enqueued, the cache and seq_len are untouched, and
 *     alora_last_error() describes the problem.
 */
#ifndef ALORA_H
#define ALORA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct alora_ctx alora_ctx;

typedef enum {
  ALORA_OK = 0,
  ALORA_EINVAL = 1,     /* null pointer, B < 1, negative length, bad option            */
  ALORA_ESHAPE = 2,     /* unsupported or inconsistent layer shape                     */
  ALORA_ECAPACITY = 3,  /* P_b + S_b exceeds the sequence's cache capacity or the pool */
  ALORA_EADAPTER = 4,   /* adapter id outside [-1, n_adapters)                         */
  ALORA_EDTYPE = 5,     /* dtype not ALORA_F32 / ALORA_BF16                            */
  ALORA_EHIP = 6        /* a HIP runtime call failed                                   */
} alora_status;

typedef enum { ALORA_F32 = 0, ALORA_BF16 = 1 } alora_dtype;

/* One decoder layer.  Immutable, caller-owned.  (Eq.2, Eq.5, Eq.6.) */
typedef struct {
  int32_t d;            /* hidden size (input width of the projections)                */
  int32_t n_q_heads;    /* query heads; must be a multiple of n_kv_heads               */
  int32_t n_kv_heads;
  int32_t head_dim;     /* even, <= 256                                                */
  int32_t rank;         /* adapter rank r, 1..256 (0 allowed when n_adapters == 0)     */
  int32_t n_adapters;   /* number of adapters stored in A / B_*                        */
  int32_t dtype;        /* alora_dtype                                                 */
  int32_t intermediate; /* SwiGLU width I; 0 = attention block only                    */
  const void *W_qkv;    /* DEVICE [N_q + 2 N_kv, d], rows ordered q | k | v            */
  const void *A;        /* DEVICE [n_adapters, 3, rank, d]   (order q, k, v)           */
  const void *B_q;      /* DEVICE [n_adapters, N_q,  rank]                             */
  const void *B_k;      /* DEVICE [n_adapters, N_kv, rank]                             */
  const void *B_v;      /* DEVICE [n_adapters, N_kv, rank]                             */
  const float *scale;   /* HOST   [n_adapters]: s_a                                    */
  const void *rms_gain; /* DEVICE [d], or NULL: no RMSNorm before the projections      */
  float rms_eps;
  float rope_theta;
  /* Rest of the layer, used by alora_stack_prefill and alora_stack_decode only (may be NULL
   * otherwise): h = x + W_o attn; out = h + W_down( silu(W_gate n) * (W_up n) ),
   * n = RMSNorm(h; rms2_gain).                                                       */
  const void *W_o;      /* DEVICE [d, N_q]                                             */
  const void *rms2_gain;/* DEVICE [d]                                                  */
  const void *W_gate;   /* DEVICE [I, d]                                               */
  const void *W_up;     /* DEVICE [I, d]                                               */
  const void *W_down;   /* DEVICE [d, I]                                               */
  /* Optional adapters of those linears (Section 2, remark after Eq.6: MLP blocks can be adapted
   * "via directly corresponding equations"; Proposition 1's proof covers them): the same rank,
   * scales and per-row gating (adapter >= 0 and position >= k) as q, k, v.  Each group is either
   * given completely or NULL (that linear stays the base model's).  alora_stack_prefill / alora_stack_decode only. */
  const void *A_o;      /* DEVICE [n_adapters, rank, N_q]                               */
  const void *B_o;      /* DEVICE [n_adapters, d, rank]                                 */
  const void *A_gu;     /* DEVICE [n_adapters, 2, rank, d]   (order gate, up)           */
  const void *B_gate;   /* DEVICE [n_adapters, I, rank]                                 */
  const void *B_up;     /* DEVICE [n_adapters, I, rank]                                 */
  const void *A_down;   /* DEVICE [n_adapters, rank, I]                                 */
  const void *B_down;   /* DEVICE [n_adapters, d, rank]                                 */
} alora_layer_desc;

/* KV cache of one layer (Eq.3: the stored K_{1:t}, V_{1:t}).  A flat pool of token rows;
 * sequence b owns rows [seq_offset[b], seq_offset[b] + seq_capacity[b]); its row j holds
 * the key / value of absolute position j.  Keys are stored after rotation.  The regions of the
 * sequences of one call must not overlap, and no sequence may write into rows that any sequence of
 * the call reads as its shared prefix (ALORA_ECAPACITY otherwise).
 *
 * Shared prefix (Section 2, "Cache reuse patterns", third regime; Proposition 2 for N adapters on one
 * context): when prefix_len is given, positions [0, prefix_len[b]) of sequence b are READ from
 * pool rows prefix_offset[b] + j -- one physical copy that any number of sequences may name, for
 * instance the rows of the base model's own sequence -- and only positions >= prefix_len[b] live
 * in the sequence's own rows, position j at seq_offset[b] + (j - prefix_len[b]).  seq_len stays
 * the full cached length (prefix included); the capacity bounds the own rows.  A call never
 * writes prefix rows (new positions are >= seq_len >= prefix_len); the caller must not hand the
 * same rows to another sequence of the same call as rows to be written.
 * The shared rows are also WALKED once: sequences of a call that name the same (prefix_offset,
 * prefix_len) put their new rows into common workgroups for the prefix keys -- in a decode step any
 * such sequences, up to 16 query-head rows per workgroup; in a prefill sequences that are neighbours
 * in the batch, up to 256 query-head rows -- so a caller keeps the sequences of one context next to
 * each other.  Results do not depend on it beyond the summation order of the attention (see
 * "Summation order" at alora_set_option). */
typedef struct {
  void *k;                     /* DEVICE [pool_tokens, n_kv_heads, head_dim]           */
  void *v;                     /* DEVICE [pool_tokens, n_kv_heads, head_dim]           */
  int64_t pool_tokens;
  const int64_t *seq_offset;   /* HOST [B]                                             */
  const int32_t *seq_capacity; /* HOST [B]                                             */
  int32_t *seq_len;            /* HOST [B]  in: P_b (rows already valid)
                                            out: P_b + S_b, written only on ALORA_OK   */
  const int64_t *prefix_offset;/* HOST [B], or NULL when prefix_len is NULL            */
  const int32_t *prefix_len;   /* HOST [B], or NULL: no sequence has a shared prefix;
                                  0 <= prefix_len[b] <= seq_len[b]                     */
} alora_kv_cache;

/* Context: create on the device that holds the buffers.  Returns ALORA_EHIP if the device
 * cannot be used.  device = -1 creates a validation-only context that needs no GPU: calls on
 * it check their arguments as usual and then return ALORA_EHIP instead of launching.
 * alora_destroy(NULL) is a no-op; destroy synchronises the device. */
alora_status alora_create(alora_ctx **ctx, int device);
void alora_destroy(alora_ctx *ctx);
/* Text of the last error on this context ("" if none); valid until the next call. */
const char *alora_last_error(const alora_ctx *ctx);
const char *alora_status_string(alora_status s);

/* Kernel selection and tuning knobs, by name.  Unknown key or value out of range: ALORA_EINVAL.
 * Every setting computes the same operation; defaults are what the benchmarks run.
 *
 *   "kernels"         0 (default): MFMA kernels for bf16 where the shape allows, plain fp32-FMA kernels
 *                     otherwise.  1: force the plain kernels (any dtype, any shape).
 *   "kv_splits"       0 (default): automatic.  n in 1..256: split the key axis of attention into n chunks
 *                     (partial results are merged by log-sum-exp weights).
 *   "gemm_splits"     0 (default): the reduction axis of every linear is cut into a number of equal segments
 *                     fixed by the shape of its weight matrix.  n in 1..64: into n segments (where the
 *                     reduction length allows; 1 = a single running sum).  See "Summation order" below.
 *   "gemm_tile"       0 (default): automatic block shape.  1: 128x128, 2: 256x128, 3: 256x256, 4: 128x64
 *                     (four waves); 5 / 6: 128x128 on eight waves of 32x64 / 64x32.  1 and 4..6 also apply to
 *                     the other linears of a stack.  A tuning experiment: with a value other than 0 the
 *                     summation-order guarantee below does not hold.
 *   "prep_split"      1 (default): calls without any adapter, with 512 rows or more at hidden size 4096 (a
 *                     base-model prefill), normalise their rows in a row-per-wave kernel; shorter calls and
 *                     calls with adapters use the kernel that prepares 16 rows per workgroup.  0: never, 2: at any
 *                     number of rows.  The normalised rows are bit-identical either way.
 *   "lora_split"      0 (default): automatic.  1: always, 2: never give the low-rank term of the QKV
 *                     projection workgroups (and a partial sum) of its own.
 *   "rope_fuse"       1 (default): where the shape allows (more than 256 rows, head size 128) the QKV
 *                     projection rotates q and k and appends k and v in its own epilogue.  0: a separate
 *                     kernel does, from the fp32 projection.  Same bits either way.
 *   "attn_waves"      0 (default) / 8: eight waves per workgroup in the prefill attention kernel.  4: four.
 *   "attn_lazy"       0..16 (default 3): the running row maximum of the prefill attention kernels moves only
 *                     when a block of scores exceeds it by more than this many powers of two (0 = exact
 *                     maximum).  The softmax is the same; only the scale of the intermediate probabilities
 *                     changes.
 *   "attn_fold"       1 (default): the queries are multiplied by log2(e)/sqrt(h) when they are written and the
 *                     score accumulators of the prefill attention kernel start at minus the row's reference
 *                     exponent, so the scores leave the matrix unit ready for exp2.  0: the kernel scales and
 *                     subtracts on the vector ALU.  The same softmax of Eq.1 either way.
 *   "attn_partials16" 1 (default): when prefill attention is split over the keys, the partial results travel
 *                     as compact records (accumulators scaled to [-1, 1] as fp16 plus three fp32 scalars,
 *                     272 bytes).  0: fp32 records (520 bytes).
 *   "stage_copy"      0 (default): the per-call records (sequences, work lists) go from the pinned host ring to
 *                     device memory by a small kernel on the call's stream.  1: by hipMemcpyAsync.
 *   "profile"         0 (default) / 1: see alora_profile_read.
 *
 * Summation order (Proposition 1 in its strong form: rows before the invocation index are the base model's
 * rows).  With "gemm_tile" = 0 the key and value rows a call appends are a function of the row's own input and
 * position alone: bit-identical whether the row came in a long prefill, a short one, a decode step, alone or
 * in a mixed batch, with or without an adapter active on OTHER rows -- every linear adds the products of a row
 * in one fixed order (segments fixed by the weight shape, each summed from zero, the sums added in ascending
 * order).  Rows before k_b of an adapter call are therefore bitwise the rows a base-only call writes.  What
 * is NOT bit-stable across differently shaped calls: attention outputs (the key axis is split by a heuristic
 * that looks at the whole batch, and prefill and decode attention are different kernels), and with them the
 * hidden states and cache rows of layers after the first in alora_stack_prefill; those agree to rounding. */
alora_status alora_set_option(alora_ctx *ctx, const char *key, int value);

/* Per-kernel timing.  With option "profile" = 1 the library brackets every kernel it launches
 * with HIP events on the call's stream.  alora_profile_read waits for the pending events and
 * returns the accumulated time and launch count of one kernel family: "prep_rows",
 * "qkv_gemm", "rope_append", "attn_prefill", "attn_decode", "attn_merge", "o_proj",
 * "mlp_norm", "gate_up", "silu_mul", "down_proj", "lm_head", "lm_argmax".  alora_profile_reset
 * clears the totals. */
alora_status alora_profile_read(alora_ctx *ctx, const char *kernel, double *total_ms, int64_t *launches);
alora_status alora_profile_reset(alora_ctx *ctx);

/* Adapter-activated prefill (Section 2, Eq.6; cost model of Proposition 2: only the T new
 * rows are projected, and each attends over its sequence's cached-plus-new rows).
 *   x_suffix        DEVICE [T, d]: hidden states of the new tokens, sequences back to back
 *   cu_seqlens      HOST [B+1]: cu[0] = 0, non-decreasing, cu[B] = T; S_b = cu[b+1]-cu[b]
 *   k_per_seq       HOST [B]: invocation index k_b >= 0
 *   adapter_per_seq HOST [B]: adapter id, or -1 for base only
 *   attn_out        DEVICE [T, N_q]: attention output of the new rows (before W_o)
 * Effects: cache rows [P_b, P_b + S_b) of every sequence are written; rows before P_b are
 * not touched (they are bit-identical afterwards); seq_len[b] += S_b.  Sequences with
 * S_b = 0 are allowed and left alone.  T = 0 is a valid no-op. */
alora_status alora_prefill(alora_ctx *ctx, const alora_layer_desc *layer, alora_kv_cache *cache,
                           const void *x_suffix, const int32_t *cu_seqlens,
                           const int32_t *k_per_seq, const int32_t *adapter_per_seq, int32_t B,
                           void *attn_out, void *stream);

/* One decode step (Eq.3-4 with the rows of Eq.6): one new token per sequence.  Same result
 * as alora_prefill with every S_b = 1, but attention runs through the memory-bound
 * split-K kernel.   x_tok DEVICE [B, d]; attn_out DEVICE [B, N_q]. */
alora_status alora_decode(alora_ctx *ctx, const alora_layer_desc *layer, alora_kv_cache *cache,
                          const void *x_tok, const int32_t *k_per_seq,
                          const int32_t *adapter_per_seq, int32_t B, void *attn_out, void *stream);

/* alora_decode for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and -- bit for bit -- the same results as
 * alora_decode, but the call allocates nothing, frees nothing, synchronises nothing and copies nothing from host
 * memory: its workspace, the per-sequence records (passed to the device as kernel arguments), the decode work
 * list and the rotary lines of the new rows live in one static device array of 32 MiB (33554432 bytes) that every
 * GPU the library runs on holds until the process ends.  A call that needs more (roughly: 5 fp32 copies of the
 * [B, N_q + 2 N_kv] projection plus B * n_q_heads * key-splits partial attention records; 64 sequences of the
 * 8B-class shape over 16k-token caches take 14 MiB) is rejected with ALORA_ECAPACITY before anything is launched,
 * as is B > 4096.  Shared prefixes are not taken (ALORA_EINVAL); the "profile" option is ignored.  All calls on
 * one GPU -- from any context, stream or thread -- share that GPU's array and it keeps the last call's contents:
 * calls that overlap in time on one GPU race, so serialise them (one stream, or events).  Nothing in the array
 * has to start at zero, and nothing is cleared.  Captured into a graph, the call's host-side effects (the checks,
 * seq_len[b] += 1) happen once, at capture; a replay repeats the captured step -- same positions, same cache rows
 * written -- on whatever the input buffer holds then.  The other entry points stage metadata through pinned host
 * slots guarded by events and may grow their workspace: do not capture those. */
alora_status alora_decode_static(alora_ctx *ctx, const alora_layer_desc *layer, alora_kv_cache *cache,
                                 const void *x_tok, const int32_t *k_per_seq,
                                 const int32_t *adapter_per_seq, int32_t B, void *attn_out, void *stream);

/* A run of n_steps decode steps (the short generations of an adapter: Section 3 times 16-token
 * evaluations) with the per-sequence arrays validated and staged once: the same result as n_steps
 * alora_decode calls, step t reading x_steps[t] and writing attn_out[t], every sequence growing by
 * one cache row per step.  For callers that already hold the inputs of all steps (teacher forcing,
 * replay, benchmarks); a sampling loop that needs the output of step t to build step t+1 calls
 * alora_decode.   x_steps DEVICE [n_steps, B, d]; attn_out DEVICE [n_steps, B, N_q];
 * seq_len[b] += n_steps; P_b + n_steps must fit the capacity. */
alora_status alora_decode_steps(alora_ctx *ctx, const alora_layer_desc *layer, alora_kv_cache *cache,
                                const void *x_steps, const int32_t *k_per_seq,
                                const int32_t *adapter_per_seq, int32_t B, int32_t n_steps,
                                void *attn_out, void *stream);

/* First-token pass through a stack of decoder layers (Proposition 2: the attention block as
 * in alora_prefill, then the per-token output projection and SwiGLU MLP with residuals -- with
 * the base weights, or gated like q, k, v where the layer carries adapters for them -- layer
 * after layer).  layers[l] must all have the same shape, dtype, rms_eps and rope_theta and carry
 * W_o / rms2_gain / W_gate / W_up / W_down.  The adapter scales s_a are taken from layers[0].scale for the whole
 * stack.  caches[l] is layer l's cache; the sequence layout (seq_offset, seq_capacity, seq_len,
 * prefixes) is read from caches[0] and applies to every layer; only caches[0].seq_len is updated.
 *   x        DEVICE [T, d]  input hidden states of the new tokens (not modified)
 *   out      DEVICE [T, d]  hidden states after the last layer                         */
alora_status alora_stack_prefill(alora_ctx *ctx, const alora_layer_desc *layers, int32_t n_layers,
                                 alora_kv_cache *caches, const void *x, const int32_t *cu_seqlens,
                                 const int32_t *k_per_seq, const int32_t *adapter_per_seq,
                                 int32_t B, void *out, void *stream);

/* One decode step through the same stack (Eq.4 in every layer: one new token per sequence over its whole
 * cache; Section 3 lets an adapter generate 16 tokens after its first): alora_stack_prefill with one row per
 * sequence, the attention of every layer running in the streaming decode kernel of alora_decode.
 *   x_tok    DEVICE [B, d]  hidden state (embedding) of each sequence's new token
 *   out      DEVICE [B, d]  hidden states after the last layer (alora_lm_head turns them into tokens) */
alora_status alora_stack_decode(alora_ctx *ctx, const alora_layer_desc *layers, int32_t n_layers,
                                alora_kv_cache *caches, const void *x_tok, const int32_t *k_per_seq,
                                const int32_t *adapter_per_seq, int32_t B, void *out, void *stream);

/* The first token itself (Section 3 times the adapter up to its first generated token): final
 * RMSNorm, projection on the vocabulary with the base model's (never adapted) output matrix, and
 * the greedy choice.  logits[b, v] = < RMSNorm(x_last[b]; final_gain), W_vocab[v] >, accumulated
 * in fp32; token[b] = the index of the largest logit, the lowest index among equals.
 *   x_last     DEVICE [B, d]      hidden state of the last new token of every sequence (dtype)
 *   final_gain DEVICE [d] or NULL (no normalisation)
 *   W_vocab    DEVICE [vocab, d]  (dtype)
 *   logits     DEVICE [B, vocab] fp32, or NULL: kept in the context workspace
 *   token      DEVICE [B] int32, or NULL: logits only
 * Sampling other than greedy is the caller's (from logits).  Same error behaviour as the calls
 * above: arguments are checked first, nothing is launched on error. */
alora_status alora_lm_head(alora_ctx *ctx, alora_dtype dtype, int32_t d, int32_t vocab, const void *x_last,
                           const void *final_gain, float rms_eps, const void *W_vocab, int32_t B,
                           float *logits, int32_t *token, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ALORA_H */
