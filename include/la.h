/*
 * liblookahead -- the lookahead-decoding verification step on one MI355X (gfx950).
 *
 * One step pushes a small block of candidate tokens (one real next-token row, W(N-1)
 * lookahead-window rows, G(N-1) n-gram verification rows) through a Mistral-family layer
 * stack against a growing KV cache, under an explicit per-row visibility mask, then
 * unembeds every row, takes the greedy argmax and accepts the longest confirmed n-gram.
 * Paper: "Privacy-Aware Split Inference with Speculative Decoding for LLMs over WANs",
 * Section 3.1 (layer partition, model shapes), 3.3 (KV cache on the side that owns the
 * layers; crop, relocation, custom masks), 4.1 (sequential step), 4.3 (lookahead decoding),
 * 4.4 (explicit masks for multi-token steps), 6.5 (output identical to greedy decoding).
 * The paper's local/cloud halves are layer ranges of one model here; its WAN transport is
 * not part of this library.  The fields its frame header carries (Section 3.2: tensor
 * shapes, cache crop position, mask) are arguments of la_forward_layers / la_ngram_accept.
 *
 * Conventions
 *  - Every function returns LA_OK (0) or a negative la_status; none throws or exits.
 *    la_last_error() gives the text of the calling thread's last failure.
 *  - "device" pointers are HIP device memory owned by the caller and borrowed for the
 *    call (the work is enqueued on `stream`; the memory must stay valid until the stream
 *    has run it).  "host" pointers are ordinary process memory, read or written before the
 *    call returns.  Handles (la_model, la_kv, la_pool) are owned by the library until freed.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *    enqueue work and do not synchronise unless stated.
 *  - Matrices are row-major [in, out].  dtype LA_F32: weights and cache are float;
 *    LA_BF16: weights and cache are bfloat16 bit patterns; LA_F16: weights, embedding table
 *    and cache are IEEE half precision (the storage type of the paper's models, Section
 *    6.1): the weight matrices are then multiplied exactly as stored and the attention
 *    multiplies q, K, V and the probabilities in half precision instead of bfloat16.  The residual stream (`hidden`),
 *    norm gains, softmax and all accumulations are float in both cases.  In LA_BF16 the
 *    weight matrices are multiplied as IEEE half precision (a bfloat16 weight of magnitude
 *    2^-14 or more converts without loss, smaller ones to within 2^-25) with activations
 *    rounded to half precision (values beyond +-65504 saturate); attention multiplies in
 *    bfloat16.
 *  - Errors raised on the device.  Two conditions are only known to a kernel: a block that
 *    does not fit the cache at the device-side length (the launch is then skipped as a
 *    whole), and a grid barrier of the persistent kernel that gave up waiting (its results
 *    are invalid).  The kernel records the code in the model's device error word and in a
 *    word of pinned host memory.  Every later call that takes the model or one of its
 *    caches looks at the host word first, without synchronising, and if it is set returns
 *    LA_ERANGE / LA_EHIP once instead of doing its work; la_kv_get_len, which synchronises,
 *    reports it for certain.  la_ngram_accept copies the device word into
 *    la_step_state.error.  After the report the next launch clears the word and the barrier
 *    state, so the model stays usable.
 *  - One stream at a time.  A la_model carries scratch memory (operand buffers, barrier
 *    words, RoPE table) that every launch on it uses: a model, and the caches made for it,
 *    may be in use on one stream at a time; two models are independent.  The persistent
 *    kernel of the matrix-core path waits at grid barriers for all of its workgroups, so
 *    it needs the GPU's compute units free of other long-running kernels while it runs.
 *    Free every la_kv before the la_model it was made for.
 *  - A block has Bp <= LA_MAX_ROWS rows.  Row b sits at cache row L+b while the block is
 *    in flight, where L is the committed cache length kept on the device inside la_kv.
 */
#ifndef LA_H
#define LA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LA_MAX_ROWS 64

typedef enum {
  LA_OK = 0,
  LA_EINVAL = -1, /* bad shape, NULL pointer, Bp out of range, unsupported combination */
  LA_ENOMEM = -2, /* device or host allocation failed */
  LA_ERANGE = -3, /* the block would not fit: L + Bp > max_len, or layer out of range */
  LA_EHIP = -4    /* a HIP call failed, or a grid barrier gave up; la_last_error() has its text */
} la_status;

typedef enum { LA_F32 = 0, LA_BF16 = 1, LA_F16 = 2 } la_dtype;

typedef struct la_model la_model; /* packed weights + per-model scratch */
typedef struct la_kv la_kv;       /* K,V cache of all layers of one model + committed length */
typedef struct la_pool la_pool;   /* n-gram pool */

/* Model shape (Section 3.1 gives layer counts, hidden size, GQA head counts, vocabulary). */
typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rms_eps, rope_theta;
  int32_t dtype; /* la_dtype */
} la_model_desc;

/* One layer's weights, device pointers, row-major [in, out], storage type = model dtype:
 * wq [d, Hq*dh], wk, wv [d, Hkv*dh], wo [Hq*dh, d], wgate, wup [d, F], wdown [F, d];
 * norm gains g_attn, g_mlp [d] are always float. */
typedef struct {
  const void *wq, *wk, *wv, *wo, *wgate, *wup, *wdown;
  const float *g_attn, *g_mlp;
} la_layer_weights;

/* Lookahead parameters (Section 4.3; the paper's "n-gram size" is N): window width W,
 * n-gram size N, at most G candidates verified per step.  Real rows per block:
 * 1 + (W + G)(N - 1) <= LA_MAX_ROWS.  {W=0, N=1, G=0} is sequential decoding (Section 4.1). */
typedef struct {
  int32_t W, N, G;
} la_lookahead_desc;

/* Controller state, resident on the device between steps (the caller allocates
 * sizeof(la_step_state) bytes of device memory; la_state_init fills it).
 *   L        committed cache length = position of c0
 *   c0       last committed token, row 0 of the next block
 *   tok/pos/vis  the block to run next: token, position and visibility mask of each of the
 *            Bp rows (bit j of vis[b]: row b attends to block row j; committed cache rows
 *            are always visible)
 *   win      lookahead window, win[r*W + c], r < N-1, c < W
 *   cand     candidates being verified in this block, cand[k*(N-1) + j], k < n_cand
 *   counters: steps, steps with at least one candidate token accepted, tokens emitted so
 *            far, and for the last step: tokens emitted, winning candidate, match length. */
typedef struct {
  int32_t L, c0, n_cand, Bp;
  int32_t steps, matched_steps, n_emitted, last_emitted, last_k, last_m;
  int32_t error, reserved;
  int32_t tok[LA_MAX_ROWS];
  int32_t pos[LA_MAX_ROWS];
  uint64_t vis[LA_MAX_ROWS];
  int32_t win[LA_MAX_ROWS];
  int32_t cand[LA_MAX_ROWS];
} la_step_state;

/* ---- model -------------------------------------------------------------------------- */

/* Creates a model and packs its weights into the library's own layout (the caller may
 * free its copies once `stream` has run).  `layers` is a host array of n_layers structs
 * of device pointers, or NULL to add layers later with la_model_set_layer.  embed [V, d],
 * unembed [d, V] (model dtype) and g_final [d] (float) are device pointers; each may be
 * NULL if la_embed / la_unembed_argmax will not be called.
 * LA_EINVAL: a dimension is not positive, Hq is not a multiple of Hkv, head_dim is odd or
 * above 256, or the GPU cannot keep the persistent kernel's workgroups (one per compute unit)
 * resident at once.
 * Two kernel paths exist.  LA_BF16 models run on the matrix-core path when d_model is a
 * multiple of 64 and at most 8192, Hq*dh and d_ffn are multiples of 32, (Hq + 2 Hkv)*dh and
 * vocab are multiples of 16, head_dim is 64 or 128 and Hq / Hkv <= 8.  Every other model
 * (LA_F32, or LA_BF16 of another shape) runs on plain kernels with float arithmetic and the
 * same results within the stated tolerance, far slower: they are the correctness path, not a
 * performance path.  The first la_forward_layers after weights were set synchronises
 * `stream` once (the table of norm-gain pointers is uploaded from pageable host memory). */
int la_init_model(const la_model_desc *desc, const la_layer_weights *layers, const void *embed,
                  const float *g_final, const void *unembed, void *stream, la_model **out);
int la_model_set_layer(la_model *m, int layer, const la_layer_weights *w, void *stream);
void la_free_model(la_model *m);

/* ---- KV cache (Section 3.3) ----------------------------------------------------------- */

/* Cache for all layers of `m`: per layer K and V of max_len rows [Hkv, dh] in the model
 * dtype, keys stored after RoPE.  max_len must leave room for the in-flight block:
 * la_forward_layers needs L + Bp <= max_len.  The committed length L starts at 0.
 * LA_EINVAL on the matrix-core path if one layer's K rows would reach 2 GiB
 * (max_len * Hkv * dh * 2 bytes: about 1M rows at Hkv*dh = 1024). */
int la_kv_alloc(const la_model *m, int max_len, la_kv **out);
/* Sets L (the paper's cache crop: rows >= L are dead). */
int la_kv_set_len(la_kv *kv, int L, void *stream);
/* Reads L back; synchronises `stream`. */
int la_kv_get_len(la_kv *kv, int *L_host, void *stream);
/* Writes n rows [n, Hkv, dh] (device, model dtype, row-major) to rows row0.. of one layer. */
int la_kv_fill(la_kv *kv, int layer, int row0, const void *k, const void *v, int n, void *stream);
/* Reads n rows starting at row0 of one layer back into row-major [n, Hkv, dh] device buffers. */
int la_kv_read(la_kv *kv, int layer, int row0, int n, void *k_out, void *v_out, void *stream);
void la_free_kv(la_kv *kv);

/* ---- the step ------------------------------------------------------------------------- */

/* hidden[b, :] = embed[tok[b], :] for b < Bp (Section 4.1 step 1).  tok: device int32 [Bp],
 * hidden: device float [Bp, d].  Token ids outside [0, vocab) are clamped. */
int la_embed(la_model *m, const int32_t *tok, int Bp, float *hidden, void *stream);

/* Runs the block through layers [layer_begin, layer_end) in place (Section 4.1 step 3 for
 * one row; Sections 3.3 / 4.4 for a block): per layer RMSNorm, QKV projection, RoPE at
 * pos[b], write of the block's K,V to cache rows L..L+Bp-1, grouped-query attention of row
 * b over {cache rows < L} U {block rows j with bit j of vis[b]}, output projection +
 * residual, RMSNorm, SwiGLU MLP + residual.
 * hidden: device float [Bp, d], in/out.  pos: device int32 [Bp].  vis: device uint64 [Bp];
 * every row must see at least itself.  Does not change L.
 * LA_EINVAL: Bp not in 1..LA_MAX_ROWS or a NULL pointer; LA_ERANGE: layer range outside the
 * model, or the host-side bound on L plus Bp exceeds max_len. */
int la_forward_layers(la_model *m, int layer_begin, int layer_end, float *hidden, int Bp,
                      const int32_t *pos, const uint64_t *vis, la_kv *kv, void *stream);

/* ids[b] = argmax_v (rmsnorm(hidden[b]) * g_final) . unembed[:, v], ties to the lowest v
 * (Section 4.1 step 5; Section 6.5: greedy argmax).  ids: device int32 [Bp].  top2: device
 * float [Bp, 2] receiving the largest and second-largest logit of each row, or NULL. */
int la_unembed_argmax(la_model *m, const float *hidden, int Bp, int32_t *ids, float *top2,
                      void *stream);

/* la_unembed_argmax for callers that cannot allocate device memory (code under HIP graph
 * capture, serving loops and harnesses that forbid hipMalloc): same arguments, same kernel
 * and bit-identical results, but the kernel's scratch memory (barrier words, the f16 operand
 * of the normalised rows, row statistics, partial arg-max records) is a static device array
 * of 4.1 MiB that every GPU the library runs on holds until the process ends, instead of
 * buffers owned by the model.  The call allocates nothing and frees nothing; it launches one
 * small fill kernel that clears the barrier words, then the unembedding kernel.
 * Only for LA_BF16 models on the matrix-core path; limits: d_model <= 8192 and
 * 256 * ceil(vocab / 4096) <= 4096 partial records (vocab <= 65536 on a 256-CU GPU), beyond
 * which it returns LA_ERANGE; LA_EINVAL for other models.  All calls on one GPU share the
 * array, whatever the model: calls that overlap in time on one GPU (two streams, two host
 * threads) race and must be serialised by the caller. */
int la_unembed_argmax_noalloc(la_model *m, const float *hidden, int Bp, int32_t *ids, float *top2,
                              void *stream);

/* Prompt prefill (Section 4.1 step 1; Section 6.3 "Prefill"): runs the n tokens tok[0..n)
 * (device int32) at positions L0.. through every layer, writes cache rows L0..L0+n-1 and
 * sets L = L0 + n.  Prompts of 128 tokens or more on the matrix-core path run as one matrix
 * product per weight matrix and chunk of 1024 tokens (the weights are read once per chunk),
 * with a causal attention kernel over the cache; shorter prompts, and models on the plain
 * kernels, go through the block kernel in causal chunks of LA_MAX_ROWS rows.  Everything is
 * enqueued on `stream`; the hidden states are not returned (generation restarts from the last
 * prompt token as c0).  The first large prompt on a model allocates its buffers (about
 * 1024 x (d_model x 8 + d_ffn x 2 + Hq x dh x 4) bytes).  LA_ERANGE: L0 + n > max_len.
 * (Chunked prefill is the paper's named future work, Section 8.) */
int la_prefill(la_model *m, la_kv *kv, const int32_t *tok, int n, int L0, void *stream);

/* ---- n-gram pool and acceptance (Section 4.3) ----------------------------------------- */

/* Pool keyed by token id: per key at most G distinct (N-1)-token continuations, refreshed
 * on re-insert, least recently inserted evicted first, looked up most recent first. */
int la_pool_alloc(int vocab, int N, int G, la_pool **out);
void la_free_pool(la_pool *p);

/* Starts a generation: clears the pool and (if seed_pool) inserts every N-gram of the prompt
 * in order; sets the window to win[r][c] = prompt[(r + c) mod P], c0 = prompt[P-1], L = P-1,
 * looks up the candidates of c0 and builds the first block of Bp rows into *state.  Also sets
 * the cache length of `kv` to P-1 (the caller prefills rows 0..P-2 through
 * la_forward_layers before or after this call).  prompt: device int32 [P], P >= 1. */
int la_state_init(la_pool *p, la_kv *kv, const la_lookahead_desc *la, const int32_t *prompt, int P,
                  int Bp, int seed_pool, la_step_state *state, void *stream);

/* The accept phase of one step, all on the device: verifies the candidates against ids
 * (the argmax of every block row), emits 1..N tokens (never more than max_total -
 * state->n_emitted) to emitted[state->n_emitted..], moves the K,V rows of the accepted
 * verification rows to cache rows L+1.. in every layer and advances L (the paper's cache
 * relocation and crop), harvests W new n-grams into the pool, slides the window, looks up
 * the candidates of the new c0 and builds the next block in *state.
 * ids: device int32 [Bp]; emitted: device int32 [>= max_total]. */
int la_ngram_accept(la_pool *p, la_kv *kv, const la_lookahead_desc *la, const int32_t *ids,
                    la_step_state *state, int32_t *emitted, int max_total, void *stream);

/* ---- Jacobi decoding (Section 4.2) ---------------------------------------------------- */

/* Jacobi parallel decoding with the same five step calls, the controller swapped: a block of
 * k future positions is guessed (first guess: the last committed token), every pass runs the
 * rows {c0, y_1, .., y_(k-1)} at positions L.. under the plain causal mask (Section 4.4)
 * through la_embed / la_forward_layers / la_unembed_argmax, and la_jacobi_accept replaces the
 * guesses by the pass's arg-max ids.  The block has converged when a pass returns the guesses
 * it was given, and after k passes at the latest (pass j makes guess j final); it then commits
 * k tokens (never more than max_total - state->n_emitted): they go to emitted[], L advances
 * over the pass's cache rows, which were computed from the final tokens, and a new block starts.
 * la_step_state in this mode: n_cand = k, cand[0..k-1] = the guesses, steps = passes so far,
 * matched_steps = blocks committed, last_emitted = tokens the last pass committed (0 while the
 * block still moves), last_k = passes spent on the current block, last_m = passes the last
 * committed block took; tok/pos/vis = the next pass (rows k..Bp-1 see only themselves).
 * la_jacobi_init also sets the cache length to P-1, like la_state_init.
 * LA_EINVAL: k outside 1..Bp, Bp > LA_MAX_ROWS, NULL pointer; LA_ERANGE: P - 1 + Bp > max_len. */
int la_jacobi_init(la_kv *kv, int k, const int32_t *prompt, int P, int Bp, la_step_state *state,
                   void *stream);
int la_jacobi_accept(la_kv *kv, int k, const int32_t *ids, la_step_state *state, int32_t *emitted,
                     int max_total, void *stream);

/* Host helper: positions and visibility masks of a lookahead block whose row 0 sits at
 * position t with n_cand candidates present (no tokens involved).  pos_host [Bp],
 * vis_host [Bp] are host arrays. */
int la_lookahead_layout(const la_lookahead_desc *la, int t, int n_cand, int Bp, int32_t *pos_host,
                        uint64_t *vis_host);

/* Host helper: positions t, t+1, ... and causal masks (row i sees block rows 0..i) of a block
 * of n consecutive tokens, as a prompt chunk is run (Section 4.1 step 1: the prompt goes
 * through the same layers before generation).  pos_host [n], vis_host [n] are host arrays;
 * 1 <= n <= LA_MAX_ROWS. */
int la_causal_layout(int t, int n, int32_t *pos_host, uint64_t *vis_host);

/* Sets how many times a workgroup polls a grid barrier's release word (about a microsecond
 * per poll) before it gives up and the launch reports LA_EHIP; 0 restores the default
 * (2^21, about two seconds).  Takes effect from the next launch on the model. */
int la_set_barrier_timeout(la_model *m, unsigned polls);

/* ---- latency model of the split deployment (host arithmetic) --------------------------- */

/* Section 6.3: the wall time of a step is the network round trip plus a fixed overhead that
 * does not depend on the network (compute on both sides, serialization).  All times in
 * milliseconds, double precision, host pointers.  LA_EINVAL for negative times, a step
 * shorter than its round trip, or a zero step time. */
int la_rtt_fixed_overhead(double per_step_ms, double rtt_ms, double *fixed_ms);
/* Section 6.3, projection model: tokens per second at round-trip time rtt_ms for a decoder
 * that commits tokens_per_step tokens per step (1 for sequential decoding) with fixed
 * overhead fixed_ms:  tokens_per_step / ((rtt_ms + fixed_ms) / 1000). */
int la_rtt_project(double tokens_per_step, double rtt_ms, double fixed_ms, double *tok_per_s);
/* Section 4.2: Jacobi decoding of a block of k tokens that converges after `iterations`
 * round trips:  k / (iterations * rtt_ms / 1000). */
int la_jacobi_project(int k, double iterations, double rtt_ms, double *tok_per_s);

/* ---- diagnostics ---------------------------------------------------------------------- */

/* Per-kernel timing with HIP events on the launch stream.  While enabled every kernel
 * launch is bracketed by events (this adds gaps: use it to attribute time, not to time a
 * step).  la_profile_read synchronises, writes up to `cap` entries (kernel name, launches,
 * total milliseconds) and returns the number of distinct kernels, then clears the record. */
typedef struct {
  char name[48];
  int32_t launches;
  float total_ms;
} la_profile_entry;
int la_profile_enable(int on);
/* Restricts the bracketing to kernels of one name (NULL or "" = all kernels again). */
int la_profile_select(const char *kernel_name);
int la_profile_read(la_profile_entry *out_host, int cap);
/* A plain copy kernel (launch name "calib_copy") that reads `bytes` from src and writes them to
 * dst (device pointers, 16-byte aligned, bytes a multiple of 16): a dispatch of known HBM
 * traffic, against which hardware byte counters read for the other kernels can be scaled. */
int la_profile_copy(void *dst, const void *src, size_t bytes, void *stream);

const char *la_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LA_H */
