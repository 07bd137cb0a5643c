/*
 * spec.h - C ABI of the MI355X (gfx950) library for parallel speculative decoding (PEARL).
 *
 * One context holds a target model M_p and a draft model M_q (paper, Section 2, notations),
 * a paged KV cache per model, a cache of the draft distributions q_i that a later verification
 * reads back (Algorithm 2) and two HIP streams so that drafting and verification overlap
 * (Section 3.4).  All arithmetic of the decoding path runs in this library's
 * kernels; callers only provide device memory for the weights and the two streams.
 *
 * Conventions
 *   - every function returns 0 (SPEC_OK) or a negative SPEC_E_* code and never throws or aborts;
 *     spec_last_error() gives a message for the last failure of the calling thread.
 *   - "device" pointers are HIP device memory on the current device, "host" pointers are
 *     ordinary host memory.  Weights and streams are BORROWED: they must outlive the context.
 *   - a context is not thread-safe; calls on one context must come from one thread at a time.
 *   - uniform random numbers are inputs (host floats in [0,1)), never drawn inside the library.
 *
 * Weight layouts (all bf16)
 *   - tok_embed      : row-major [vocab][d_model]
 *   - norm gains     : [d_model]
 *   - projections    : "panel-packed" (see spec_pack_weight).  A projection y = x W^T with
 *                      W [N][K] is stored as N/16 panels; wqkv is the concatenation of the
 *                      panels of W_q, W_k, W_v; w_gateup interleaves panels (gate panel j at
 *                      2j, up panel j at 2j+1).
 */
#ifndef SPEC_H
#define SPEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  SPEC_OK = 0,
  SPEC_E_INVAL = -1, /* bad argument; nothing was changed                         */
  SPEC_E_NOMEM = -2, /* KV pages or device memory exhausted; state left unchanged  */
  SPEC_E_STATE = -3, /* call not valid in the current state (e.g. no prefill yet)  */
  SPEC_E_HIP = -4    /* a HIP call failed; the context should be freed             */
};

enum { SPEC_TARGET = 0, SPEC_DRAFT = 1 };

/* Which acceptance step to run (spec_accept). */
enum {
  SPEC_ACCEPT_AR = 0,   /* no draft: draw the next token from row 0 of the last target forward      */
  SPEC_ACCEPT_SD = 1,   /* vanilla speculative decoding, Section 2: every row but the last tests a draft,
                           the last row draws the bonus token when all are accepted                      */
  SPEC_ACCEPT_PRE = 2,  /* pre-verify, Section 3.2 / Algorithm 2: row p = M_p(x) tests x_1          */
  SPEC_ACCEPT_POST = 3, /* post-verify, Section 3.3 / Algorithm 2: every row tests a draft, no bonus.
                           For SD and POST row 0 tests x_1, or x_2 when x_1 is already committed (it then
                           was the first token of the verify forward)                                    */
  SPEC_ACCEPT_PRE_GUESS = 4 /* pre-verify of several draft tokens (closing remark of Section 4.3), after
                           spec_verify_guess: row 0 = M_p(x) tests x_1; row i >= 1 = M_p(x + [g_1..g_i]) tests
                           x_{i+1}, but only while the accepted drafts x_1..x_i are the guesses g_1..g_i - the
                           first draft that leaves the guessed path ends the step without a rejection        */
};
enum { SPEC_MODE_PRE = 0, SPEC_MODE_POST = 1 };

#define SPEC_MAX_TOKENS 32 /* most tokens one forward may take (gamma_max + 1 <= SPEC_MAX_TOKENS) */

typedef struct spec_ctx spec_ctx;

typedef struct {
  int n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rope_theta, rms_eps;
} spec_model_desc;

/* Device pointers, bf16.  Per-layer arrays are host arrays of n_layers device pointers. */
typedef struct {
  const void* tok_embed;
  const void* final_norm;
  const void* lm_head;        /* packed [vocab][d_model]                       */
  const void* const* attn_norm;
  const void* const* wqkv;    /* packed [(n_heads + 2 n_kv_heads) head_dim][d_model] */
  const void* const* wo;      /* packed [d_model][n_heads head_dim]            */
  const void* const* ffn_norm;
  const void* const* w_gateup;/* packed, gate/up panels interleaved, [2 d_ffn][d_model] */
  const void* const* w_down;  /* packed [d_model][d_ffn]                       */
} spec_weights;

typedef struct {
  int gamma_max;      /* largest window size gamma that will be used (1..SPEC_MAX_TOKENS-1) */
  int max_seq;        /* most tokens (prompt + generated + 2 gamma_max of speculation) a cache must hold */
  int page_tokens;    /* tokens per KV page: 64                                             */
  float temperature;  /* 0 = greedy (distributions become one-hot at the arg-max)           */
  float logit_scale;  /* logits are multiplied by this before the softmax                   */
  void* stream_target;/* hipStream_t, borrowed                                              */
  void* stream_draft; /* hipStream_t, borrowed; may equal stream_target (serialised).  For the two
                         passes to overlap the streams must sit on different hardware queues: plain
                         streams are dealt round-robin to a few shared queues and may end up on the
                         same one; a stream from hipExtStreamCreateWithCUMask (a mask of all compute
                         units will do) owns a queue.  Default priority only.               */
} spec_config;

/* ---- the decoding path --------------------------------------------------------------- */

/* Build a context: allocates KV pages, activation scratch, the q cache and events on the
 * current device.  Both models must have the same vocabulary.  SPEC_E_INVAL on unsupported
 * shapes (head_dim not 64/128, sizes not multiples of 16/8), SPEC_E_NOMEM if allocation fails. */
int spec_init(const spec_config* cfg, const spec_model_desc* target, const spec_weights* tw,
              const spec_model_desc* draft, const spec_weights* dw, spec_ctx** out);
void spec_free(spec_ctx* ctx);

/* Reset both caches and feed prompt[0..n-2] to both models; prompt[n-1] becomes the frontier
 * (the last committed token, the one token neither cache holds yet); mode := pre-verify.
 * This is the evaluation of both models on the prefix in Algorithm 2, done with a KV cache.  Synchronous.
 * Errors found before anything is touched (bad arguments, a prompt that cannot fit) leave the context as it
 * was; a failure after the caches have been reset leaves it un-prefilled: every decoding call then returns
 * SPEC_E_STATE until a spec_prefill succeeds.
 * `which_mask`: bit SPEC_TARGET / bit SPEC_DRAFT select the models to prefill (3 = both). */
int spec_prefill(spec_ctx* ctx, const int32_t* prompt_host, int n_prompt, int which_mask);

/* One drafting forward, asynchronous on the draft stream: q_i = M_q(x + [x_1..x_{i-1}]),
 * x_i ~ q_i by inverse CDF with the uniform u (Algorithm 2, drafting loops).  The first call
 * after an acceptance feeds the committed tokens the draft cache lacks (normally just the
 * frontier); later calls feed the previously drafted token, which never leaves the device.
 * q_i and x_i are appended to the q cache.  If tok_out_host is not NULL the call synchronises
 * and returns x_i (tests only).  SPEC_E_STATE after 2*gamma_max unverified drafts. */
int spec_draft_step(spec_ctx* ctx, float u, int32_t* tok_out_host);

/* One target forward over n_tokens tokens against the KV cache, asynchronous on the target
 * stream: the verification of several draft tokens in one forward (Section 1; rows p_1..p_n
 * of Section 2).  tokens_host == NULL selects the tokens the step needs: the frontier followed
 * by the first n_tokens-1 unverified drafts, read on the device.  If one of those drafts is
 * still being produced (vanilla SD verifies the chain it has just launched; PEARL's rows were
 * drafted in earlier steps) the call blocks the host until the draft stream has produced it and
 * only then enqueues the forward: a target stream parked on a device-side wait slows the draft
 * stream's kernel launches.  If logits_out_host is not NULL the call synchronises and copies the
 * fp32 logits [n_tokens][vocab] (tests only). */
int spec_verify(spec_ctx* ctx, const int32_t* tokens_host, int n_tokens, float* logits_out_host);

/* Pre-verify over guessed continuations - Section 4.3 ends with the remark that pre-verify could cover several
 * draft tokens with the help of a candidate pool; the paper gives no algorithm, this is the library's reading of it.
 * One target forward, asynchronous on the target stream, over the frontier x followed by guesses g_1..g_m of how
 * the text goes on: row 0 is M_p(x) as in pre-verify (Section 3.2), row i is M_p(x + [g_1..g_i]).  If the draft
 * model happens to draft x_1..x_i = g_1..g_i, row i is the target's exact distribution for x_{i+1}, so
 * spec_accept(SPEC_ACCEPT_PRE_GUESS) can test several drafts with Eq. (1) in the pre-verify step; a wrong guess
 * only wastes its row, the output distribution stays the target's.
 * guess_host != NULL: n_guess tokens from the caller's candidate pool.  guess_host == NULL: the library's pool,
 * the committed text itself as an n-gram cache - up to n_guess tokens that followed the most recent earlier
 * occurrence of the frontier token (possibly none).  0 <= n_guess <= gamma_max - 1.  *n_fed (nullable) = guesses
 * actually fed, i.e. the forward has *n_fed + 1 rows.  Needs fresh drafts (x_1 not yet committed), else
 * SPEC_E_STATE.  logits_out_host as in spec_verify. */
int spec_verify_guess(spec_ctx* ctx, const int32_t* guess_host, int n_guess, int* n_fed, float* logits_out_host);

/* Speculative-sampling accept / reject on the device (Eq. (1): accept x iff r <= p[x]/q[x];
 * on the first rejection draw from norm(max(0, p - q)); Section 2 and Algorithm 2), then the
 * bookkeeping of the step.  Waits for both streams.  r_host[0..n_r-1] are the acceptance
 * uniforms in test order, u_resample draws the corrected / bonus / autoregressive token.
 * Outputs: *n_accepted draft tokens accepted; tokens_out_host[0..*n_out-1] the tokens committed
 * by this step (at most gamma_max + 1); *next_mode the strategy of the next PEARL step.
 * After the call the frontier is the last committed token.  *keep_len is -1 when the caches stay
 * as they are (drafts still pending), otherwise the caller must cut every cache that holds more
 * than *keep_len (= committed - 1) tokens back to that length with spec_rollback_kv.
 * SPEC_ACCEPT_PRE_GUESS without a rejection commits the n >= 1 accepted drafts, keeps x_{n+1}.. pending (the next
 * post-verify forward then has fewer rows: spec_pending_rows) and itself cuts the target cache back to committed - 1
 * tokens (the guess rows behind the new frontier go; the draft cache stays): *keep_len is -1.
 * `force_mask`: < 0 = real decisions; otherwise bit i overrides the i-th decision (1 = accept)
 * - measurement and scripted tests only. */
int spec_accept(spec_ctx* ctx, int kind, const float* r_host, int n_r, float u_resample, long long force_mask,
                int* n_accepted, int32_t* tokens_out_host, int* n_out, int* next_mode, int* keep_len);

/* Drop everything after the first new_len tokens of one model's cache: O(1) - sets the length
 * and returns whole pages to the pool (the discarding of the newer drafts after a rejection in
 * Figure 3).  Unverified drafts that lie beyond the new length are forgotten.  SPEC_E_INVAL if
 * new_len > current length. */
int spec_rollback_kv(spec_ctx* ctx, int which, int new_len);

/* Forget every unverified draft token and its q row (the caller rolls the draft cache back itself). */
int spec_drop_drafts(spec_ctx* ctx);

/* Go back to the state right after the first committed_len committed tokens (prompt included):
 * later tokens and all drafts are forgotten, both caches are cut to committed_len - 1 tokens,
 * mode := pre-verify.  1 <= committed_len <= spec_committed_len(ctx), else SPEC_E_INVAL. */
int spec_rewind(spec_ctx* ctx, int committed_len);

int spec_kv_len(const spec_ctx* ctx, int which);     /* tokens currently in that model's cache */
/* Rows of the next post-verify forward: the frontier (when it is the accepted draft x_1) plus the unverified
 * drafts behind it.  gamma in Algorithm 2; 1..gamma after a pre-verify step over guesses; 0 with no drafts. */
int spec_pending_rows(const spec_ctx* ctx);
int spec_committed_len(const spec_ctx* ctx);         /* prompt + committed generated tokens    */
int spec_kv_free_pages(const spec_ctx* ctx, int which);
long long spec_forward_count(const spec_ctx* ctx, int which); /* forwards run so far by that model */

/* Whole loops on top of the calls above (host control flow only): Algorithm 1/2 (algo 2), vanilla
 * speculative decoding (algo 1), autoregressive decoding (algo 0), and the two ablations of Section 4.3:
 * PEARL without pre-verify (algo 3: after a rejection one step only drafts, then the target verifies the frontier
 * and x_1..x_gamma while the draft goes on) and without post-verify (algo 4: x_1 is verified early, then the target
 * verifies x_2..x_gamma and draws a bonus token while the draft model idles).  algo 5 is PEARL whose pre-verify
 * steps cover several draft tokens (spec_verify_guess with the library's pool, SPEC_OPT_GUESS_TOKENS guesses; with 0
 * guesses it takes exactly the steps of algo 2); its post-verify step after such a step verifies what is left of
 * the window (1..gamma rows).  Uniform arrays are indexed
 * by step: u_draft[t*gamma + i], r_accept[t*(gamma+1) + i], u_resample[t]; each must hold
 * n_generate steps (2 n_generate for algo 3, whose draft-only steps commit nothing).  The loop ends after n_generate tokens, or after max_steps steps if
 * max_steps > 0.  force_bits == NULL uses real decisions; otherwise decision (t, i) is taken
 * from force_bits[t*(gamma+1)+i] (measurement only).  SPEC_E_STATE if drafts of an earlier call are still
 * pending that this loop cannot take over (any for algo 0 / 1; a number other than gamma for the PEARL variants,
 * more than gamma for algo 5).
 * out_tokens_host receives the committed
 * tokens (at most n_generate; stats[1] tells how many were committed).
 * stats_host (nullable, 8 doubles): steps, committed, draft forwards, target forwards,
 * accepted, tested, post-verify steps, seconds. */
int spec_generate(spec_ctx* ctx, int algo, int gamma, int n_generate, int max_steps, const float* u_draft,
                  const float* r_accept, const float* u_resample, const uint8_t* force_bits,
                  int32_t* out_tokens_host, double* stats_host);

/* Window size of Section 4.4.1: gamma = round(c), c = T(one target forward) / T(one draft forward incl. its draw),
 * both over one token at the current context length, clamped to [1, min(cap, gamma_max)].
 * concurrent == 0: each model timed with the GPU to itself, n_iter forwards each (the paper's setting: one device
 * per model).  concurrent != 0: both streams busy at once, as inside a PEARL step on one GPU (needs two streams).
 * Needs a prefilled context between steps (no drafts pending, else SPEC_E_STATE); leaves caches, committed tokens
 * and mode as it found them.  Outputs: *gamma_out and the two times in seconds per forward.  Synchronous. */
int spec_calibrate_gamma(spec_ctx* ctx, int n_iter, int cap, int concurrent, int* gamma_out, double* t_target_s,
                         double* t_draft_s);

const char* spec_last_error(void);

/* ---- set-up helpers and single kernels (tests, benchmarks) ------------------------------ */

/* Repack a row-major bf16 matrix W[N][K] (device) into 16-row panels for the projection
 * kernels.  Panel j of this matrix is written as panel (panel_start + j*panel_step) of dst;
 * one panel is K_pad/32 blocks of 1 KiB (K_pad = K rounded up to 32, zero filled), block t
 * holding for lane l = 16*(kk/8) + row the eight values W[16 j + row][32 t + kk .. +7].
 * N % 16 == 0 and K % 8 == 0 are required.  Asynchronous on `stream`. */
int spec_pack_weight(void* dst_dev, const void* src_dev, int N, int K, int panel_start, int panel_step,
                     void* stream);
size_t spec_packed_bytes(int N, int K);

/* y[M][N] (fp32, device) = x[M][K] (bf16 row-major, device) * W^T with W panel-packed.
 * The same kernel the forward uses; `work_dev` needs spec_gemm_workspace_bytes(M, N, K).
 * M <= SPEC_MAX_TOKENS.  Asynchronous on `stream`. */
int spec_gemm(float* y_dev, const void* x_dev, const void* w_packed_dev, int M, int N, int K,
              void* work_dev, void* stream);
size_t spec_gemm_workspace_bytes(int M, int N, int K);
/* How that kernel divides its work (host-only, no GPU needed): out6 = { S = K slices, most K steps of 32 a wave
 * takes (at most 8), Gs = groups of workgroups along N, number of 16-row panels, number of K steps, 16-row tiles
 * of x (1 or 2) }.  workgroups_per_cu is 1 or 2; S does not depend on it.  SPEC_E_INVAL for shapes spec_gemm
 * refuses. */
int spec_gemm_plan_query(int M, int N, int K, int workgroups_per_cu, int* out6);
/* Only the streaming kernel of spec_gemm (no reduction pass); used to time it in isolation. */
int spec_gemm_partials(const void* x_dev, const void* w_packed_dev, int M, int N, int K,
                       void* work_dev, void* stream);

/* The prompt-sized projection of spec_prefill's dense path (matrix-core bound, any M >= 1):
 *   epilogue 0: y[M][N] (fp32, device)  = x[M][K] W^T
 *   epilogue 1: y[M][N] (fp32, device) += x[M][K] W^T                      (residual add)
 *   epilogue 2: z[M][N/2] (bf16, device) = silu(gate) * up, where W holds the gate and up matrices
 *               with their 16-row panels interleaved (even panel = gate, odd = up)
 * x is bf16 row-major, W panel-packed (spec_pack_weight).  N % 16 == 0 and K % 32 == 0 are required
 * (N % 32 == 0 for epilogue 2); the unused one of y / z may be NULL.  Asynchronous on `stream`. */
int spec_dense_gemm(float* y_dev, void* z_dev, const void* x_dev, const void* w_packed_dev, int M, int N, int K,
                    int epilogue, void* stream);

/* Streaming-read probe: sums `bytes` bytes of device memory with 16-byte loads; used to
 * measure the achievable HBM read ceiling next to the nominal peak.  out_dev: 4 bytes. */
int spec_read_probe(const void* src_dev, size_t bytes, void* out_dev, void* stream);

/* Fused scale -> softmax -> inverse-CDF draw on one fp32 logits row (device):
 * writes the distribution to q_out_dev[vocab] and the token to tok_out_dev[0]. */
int spec_sample_row(const float* logits_dev, int vocab, float temperature, float logit_scale, float u,
                    float* q_out_dev, int32_t* tok_out_dev, void* stream);

/* Acceptance on caller-provided rows (device): p_logits [n_rows][vocab] fp32 logits of the
 * target, q_rows [n_test][vocab] distributions, x_dev[n_test] draft tokens, r_host[n_test].
 * If n_rows == n_test + 1 and all are accepted a bonus token is drawn from the last row.
 * result_host[0] = n_accepted, result_host[1] = corrected/bonus token (or -1). Synchronous. */
int spec_accept_rows(const float* p_logits_dev, int n_rows, const float* q_rows_dev, const int32_t* x_dev,
                     int n_test, int vocab, float temperature, float logit_scale, const float* r_host,
                     float u_resample, int32_t* result_host, void* stream);

/* spec_accept_rows for callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): same arguments and the same kernels, but the kernels' scratch (row statistics, one row
 * of draw weights, the result record) lives in a device array of the library, about 1 MiB that every GPU the
 * library runs on holds until the process ends, and the outcome goes to result_dev[0..1] (device memory of the
 * caller: n_accepted, corrected / bonus token or -1).  Calls no hipMalloc / hipFree; asynchronous on `stream`.
 * vocab <= SPEC_STATIC_VOCAB_MAX, else SPEC_E_INVAL.  All calls on one GPU share the array: calls that overlap on
 * one GPU (two streams, two threads) race - serialise them. */
#define SPEC_STATIC_VOCAB_MAX 262144
int spec_accept_rows_static(const float* p_logits_dev, int n_rows, const float* q_rows_dev, const int32_t* x_dev,
                            int n_test, int vocab, float temperature, float logit_scale, const float* r_host,
                            float u_resample, int32_t* result_dev, void* stream);

/* Options.  SPEC_OPT_GEMM_WGS_PER_CU: how many workgroups of a projection kernel are launched per compute
 * unit.  2 fills both slots of every CU (fastest when a stream runs alone), 1 leaves one slot to the other
 * stream's kernels so that draft and target passes run side by side, -1 (default) = automatic: spec_generate's
 * PEARL loop on two different streams uses 1, everything else 2.  Results do not depend on it (the K split
 * and the order of additions are fixed by the shape).
 * SPEC_OPT_GRAPHS: 1 (default) = every forward is captured once per (model, token count, mode) into a HIP graph
 * and replayed; 0 = launch kernel by kernel.  Results are identical.
 * SPEC_OPT_PREFILL: how spec_prefill feeds the prompt.  1 = dense path: blocks of up to 4096 tokens go through
 * matrix-core GEMMs and a causal flash-attention kernel (needs d_model, n_heads*head_dim and d_ffn to be
 * multiples of 32, else SPEC_E_INVAL at spec_prefill); 0 = as a sequence of 32-token verify forwards (the
 * decode kernels); -1 (default) = dense when the shapes allow it and the prompt has more than 64 tokens.
 * Both fill the caches with the same K / V up to bf16 rounding of differently ordered sums.
 * SPEC_OPT_FUSE_SINGLE: 1 (default) = forwards over a single token (every draft step, autoregressive and pre-verify
 * target forwards) run seven kernels per layer: the QKV, gate/up and down projections form their input in their
 * prologue (residual add + norm input, SiLU * mul); 0 = the ten-kernel chain that forwards over several tokens use.
 * Same operations, sums in the same order up to the grouping of the sums of squares (results agree to fp32
 * rounding, not bit for bit).
 * SPEC_OPT_TARGET_TAIL_LAYERS: while the two models overlap with one projection workgroup per CU and stream (PEARL
 * loops from gamma 6 on, or SPEC_OPT_GEMM_WGS_PER_CU = 1), the last n layers of a target forward (rounded to whole
 * launch chunks of the forward) and its LM head launch with two: the chain that would end later gets the larger share
 * of the memory pipe, and what is left of it after the draft chain has ended runs at the full rate.  -1 (default):
 * spec_generate's PEARL loops move n by one chunk per step from where the two chains of the last step ended (the
 * balance the window size of Section 4.4.1 aims at, reached here at run time); n >= 0: fixed.  The results do not
 * depend on it (the K split of a projection is the same in both launch modes).  spec_get_option reads the n in use.
 * SPEC_OPT_GUESS_TOKENS: most guesses k a pre-verify step of algo 5 feeds behind the frontier; -1 (default) =
 * gamma - 1, the most that can be used; values above gamma - 1 are clipped.
 * SPEC_OPT_TEST_FAIL_PREFILL (tests of the error path only): n > 0 makes the next spec_prefill give up with
 * SPEC_E_NOMEM after its n-th forward, as if the KV pages had run out half way; one-shot.
 * spec_get_option reads a value back; for SPEC_OPT_GEMM_WGS_PER_CU it is the mode the next forward launches with
 * (1 or 2). */
enum { SPEC_OPT_GEMM_WGS_PER_CU = 1, SPEC_OPT_GRAPHS = 2, SPEC_OPT_PREFILL = 3, SPEC_OPT_TEST_FAIL_PREFILL = 4,
       SPEC_OPT_FUSE_SINGLE = 5, SPEC_OPT_GUESS_TOKENS = 6, SPEC_OPT_TARGET_TAIL_LAYERS = 7 };
int spec_set_option(spec_ctx* ctx, int option, int value);
int spec_get_option(const spec_ctx* ctx, int option, int* value);

/* Run-time switches: bit 0 = every projection launch of the target forward records its own duration: its
 * workgroups stamp the device's constant-rate wall clock on the way in and out, the earliest start and the latest end
 * are kept per launch (no dispatch overhead in it, unlike events around a launch; up to 65536 launches between two
 * reads).  Forwards are then launched kernel by kernel, not as graphs.  Read with spec_profile_read. */
int spec_set_profile(spec_ctx* ctx, int flags);
/* Sum of the recorded projection-kernel durations (ms), launch count and weight bytes since the last read. */
int spec_profile_read(spec_ctx* ctx, double* ms_total, long long* n_launches, double* bytes_total);

#ifdef __cplusplus
}
#endif
#endif /* SPEC_H */
