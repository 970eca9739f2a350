/*
 * asd.h: C ABI of the MI355X (gfx950) engine for adaptive self-speculative decoding.
 *
 * The engine runs the batch-1 Llama-style decoder two ways: as a layer-skipping
 * draft pass (one token per step, attention / MLP sublayers dropped per a skip
 * mask) and as a (k+1)-row greedy verification pass over the full model, and it
 * taps, in both, the cosine similarity between the hidden state entering and
 * leaving every sublayer.  Paper anchors: Section 1 (draft / verify / replace the
 * first rejected token), Section 3.2 (average cosine similarity C_l over the
 * prompt, CS thresholding, rules 1 and 2) and Algorithm 1 (ADMG).
 *
 * Conventions
 *   - Every function returns ASD_OK (0) or a negative ASD_E_* code; the message
 *     is available from asd_last_error().  Outputs are written only on success.
 *     No C++ exception crosses this boundary.
 *   - Pointers are HOST pointers unless the comment says DEVICE.
 *   - Device memory is caller-owned: the caller allocates one arena of
 *     asd_arena_bytes() bytes (256-byte aligned) and lends it to the engine until
 *     asd_destroy(); the engine never allocates or frees device memory.
 *   - The HIP stream is caller-owned; all work is enqueued on it.  Calls that
 *     return host data synchronise that stream before returning.
 *   - Layers are 0-based here.  A skip mask has 2L bytes: index 2l = attention
 *     sublayer of layer l, 2l+1 = its MLP; non-zero = removed from the model.
 *   - An engine is not thread-safe; calls on one engine must not overlap.
 *   - Matrices are row-major [out_features][in_features] in the storage type of
 *     the configuration (fp32, or bf16 bit patterns); norm gains are fp32.
 */
#ifndef ASD_H
#define ASD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ASD_OK = 0, ASD_E_INVAL = -1, ASD_E_STATE = -2, ASD_E_NOMEM = -3, ASD_E_IO = -4, ASD_E_HIP = -5 };

enum { ASD_DT_F32 = 0, ASD_DT_BF16 = 1 };

/* Tensor identifiers for asd_set_weight / asd_get_weight. */
enum {
    ASD_T_EMBED = 0, ASD_T_ATTN_NORM = 1, ASD_T_WQ = 2, ASD_T_WK = 3, ASD_T_WV = 4, ASD_T_WO = 5,
    ASD_T_MLP_NORM = 6, ASD_T_WG = 7, ASD_T_WU = 8, ASD_T_WD = 9, ASD_T_FINAL_NORM = 10, ASD_T_LM_HEAD = 11
};

#define ASD_MAX_ROWS 16   /* rows per forward call: draft length k <= 15 */
#define ASD_MAX_SEQ 65536  /* cache capacity in positions */

typedef struct asd_engine asd_engine;   /* opaque, library-owned host object */

/*
 * Model and cache shape.  Constraints (else ASD_E_INVAL): d_model, d_ffn, vocab,
 * n_heads*head_dim multiples of 16; head_dim 32, 64 or 128; n_heads a multiple
 * of n_kv_heads; page_tokens a multiple of 64; 1 <= max_rows <= ASD_MAX_ROWS;
 * max_seq >= 1 (rounded up to whole pages), and the rounded capacity at most
 * ASD_MAX_SEQ positions (the decode-attention merge holds the statistics of at
 * most 256 groups of 256 keys per head).
 * dtype is the storage type of weights and of the KV cache and the operand type
 * of the matrix cores (with bf16, activations go in as a hi + lo pair of bf16
 * values); the residual stream and every accumulation are fp32.
 */
typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
    int32_t max_seq, page_tokens, max_rows;
    int32_t dtype;              /* ASD_DT_F32 or ASD_DT_BF16 */
    float rms_eps, rope_theta;  /* 1e-5, 1e4 for Llama-2 */
    uint32_t debug_flags;       /* ASD_DBG_* bits; 0 in production */
    const char* debug_tune;     /* launch-shape overrides (see below); NULL in production */
} asd_config;

/*
 * Development and test switches, all explicit in the configuration (the library reads no environment
 * variable and keeps no global state).  None of them changes what is computed; the tests use them to
 * show that alternative launch shapes give the same bits.
 *   ASD_DBG_ATT_W4      always launch the decode-attention variant compiled for four waves per SIMD
 *   ASD_DBG_ATT_GH1     one query head per decode-attention workgroup also for grouped-query models
 *   ASD_DBG_RS_POW2     row stride of the activation buffers = next power of two >= rows (default: rows)
 *   ASD_DBG_SAMPLE_MEM  sampling kernels that re-read their logit rows from memory
 * debug_tune: "name=a,b,c,d;..." with name in {qkv, o, gu, down, lm}: tiles per workgroup, waves per
 * workgroup, k-major layout (0/1), interleaved k-blocks (0/1); and name in {pf_qkv, pf_o, pf_gu,
 * pf_down}: 16-row chunks per workgroup, K slices[, prefetch depth[, tiles per wave (pf_qkv: 3..5)]] of the prompt-block GEMMs;
 * "qkv_rows=N": tiles per QKV workgroup in passes of five rows and more (default: by balance).  A
 * layout override changes how weights are tiled in the arena, never their values.  The string is
 * copied by asd_create.
 */
enum { ASD_DBG_ATT_W4 = 1, ASD_DBG_ATT_GH1 = 2, ASD_DBG_RS_POW2 = 4, ASD_DBG_SAMPLE_MEM = 8 };

/*
 * Parameters of speculative generation.  alpha, m, n are Algorithm 1's inputs
 * (Table 2: 0.985, 3, 2); m = 0 switches rule 1 off, n = 0 rule 2, use_cs = 0
 * CS thresholding (the rule subsets of the ablation, Table 5).
 * draft_len = k >= 0 drafted tokens per cycle (0 = plain greedy decoding).
 * mask_mode 0: skip mask = ADMG of the prompt's ACS (the paper's method);
 * mask_mode 1: fixed_mask [2L] is used as given;
 * mask_mode 2: as 0, then the mask is rebuilt after every verification pass from
 *   the running ACS over the prompt rows and all rows committed since (the
 *   verification pass is a full-model pass, so its accepted rows extend the average
 *   that Section 3.2 defines as C_l); an extension, the paper builds the draft model once per prompt.
 * use_graphs != 0 replays each draft/verify cycle as a captured HIP graph.
 * use_cs_mlp != 0 also removes MLP sublayers whose ACS reaches alpha_mlp (subject
 *   to rule 2); an extension, Algorithm 1 thresholds attention sublayers only.
 * exit_mode 0: every cycle drafts draft_len tokens (fewer only at the end).
 * exit_mode 1: adaptive draft exit (Section 4 takes it from the Draft & Verify
 *   paper and prints neither the rule nor its constants, so all constants are
 *   the caller's): a cycle stops drafting after a token whose softmax probability
 *   under the draft model is below gamma (that token is still verified), at
 *   draft_len tokens at the latest; after a verification that accepted a of d
 *   drafts, AR <- beta1*AR + (1-beta1)*a/d, gamma~ = gamma + eps if AR <= ar_target
 *   else gamma - eps, gamma <- beta2*gamma + (1-beta2)*gamma~, starting from
 *   gamma0, ar0.  The host decides, in double, on the fp32 probability the device
 *   computed; one device-to-host read per draft step.
 * temperature 0: greedy decoding; whatever the fields above say, the emitted tokens
 *   equal plain greedy decoding of the full model.
 * temperature > 0: sampled decoding from softmax(logits / temperature).  Section 1 cites
 *   the speculative-sampling rule for it without printing it: a draft x ~ q is kept with
 *   probability min(1, p(x)/q(x)), the first rejected draft is replaced by a draw from the
 *   normalised residual max(0, p - q), and when all drafts are kept one more token is
 *   drawn from the full model; the emitted tokens are then distributed as samples of the
 *   full model alone.  Uniforms are counter based on `seed`: output index e uses
 *   U(e, c) = (mix64(stream + (3e + c + 1) * GOLD) >> 11) * 2^-53, c = 0 draft draw,
 *   1 accept test, 2 replacement / extra / plain draw, with the synthetic-input
 *   generator's stream key for tensor id 102.  asd_generate draws the prompt pass's
 *   token with U(0, 2) and decodes from index 1; asd_decode starts at sample_index0.
 *   exit_mode must be 0.
 */
typedef struct {
    float alpha;
    int32_t m, n, use_cs;
    int32_t draft_len;
    int32_t mask_mode;
    const uint8_t* fixed_mask;
    int32_t use_graphs;
    float alpha_mlp;
    int32_t use_cs_mlp;
    int32_t exit_mode;
    double gamma0, ar0, ar_target, eps, beta1, beta2;
    float temperature;
    uint64_t seed;
    int64_t sample_index0;
} asd_gen_params;

/* Counters of one asd_decode / asd_generate call (emitted includes the first token for asd_generate);
 * gamma, ar: final values of the adaptive draft exit; mask_changes: rebuilds that changed the mask.
 * ms_decode is host wall time of the whole decode call.  ms_draft / ms_verify are GPU time of the draft
 * passes and of the verification passes (accept / rollback included), from HIP events recorded on the
 * engine's stream between the phases of every cycle; ms_other = ms_decode - ms_draft - ms_verify (host
 * decisions, the per-cycle read of the decoding state, idle gaps).  bytes_draft / bytes_verify are the
 * algorithmic bytes those passes had to read (kept sublayers' weights, LM head, K/V of the visible
 * context), summed over the call. */
typedef struct {
    int64_t cycles, drafted, accepted, emitted;
    double ms_prefill, ms_decode;
    int64_t mask_changes;
    double gamma, ar;
    double ms_draft, ms_verify, ms_other;
    double bytes_draft, bytes_verify;
} asd_gen_stats;

/* Per-kernel-class GPU time of one profiled forward pass, from HIP events on the engine's stream. */
enum { ASD_K_EMBED = 0, ASD_K_QKV = 1, ASD_K_ATTN = 2, ASD_K_OPROJ = 3, ASD_K_GATEUP = 4,
       ASD_K_DOWN = 5, ASD_K_LMHEAD = 6, ASD_K_FINISH = 7, ASD_K_COUNT = 8 };
typedef struct {
    double ms[ASD_K_COUNT];       /* summed duration of the launches of each class */
    int32_t launches[ASD_K_COUNT];
    double bytes[ASD_K_COUNT];    /* algorithmic bytes those launches must read (weights, KV) */
    double ms_total;              /* first launch start to last launch end */
} asd_kernel_times;

/* Bytes of device memory the engine needs for this configuration (0 if the configuration is invalid). */
size_t asd_arena_bytes(const asd_config* cfg);

/*
 * Create an engine on the current HIP device.  device_arena: DEVICE pointer to
 * arena_bytes >= asd_arena_bytes(cfg) bytes, 256-byte aligned, borrowed until
 * asd_destroy.  hip_stream: a hipStream_t (NULL = the default stream).
 * The KV cache and workspace are cleared; weights are unset.
 */
int asd_create(const asd_config* cfg, void* device_arena, size_t arena_bytes, void* hip_stream, asd_engine** out);
void asd_destroy(asd_engine* e);

/* Message of the last failing call on this engine (or of the last failing asd_create when e is NULL). */
const char* asd_last_error(const asd_engine* e);

/*
 * Weights.  asd_set_weight copies one tensor (bytes must match its size) from host
 * or, when src_on_device != 0, from DEVICE memory, and re-tiles matrices into the
 * engine's streaming layout.  asd_get_weight returns it to HOST memory, row-major.
 * asd_init_synthetic fills every tensor on the device with the counter-based
 * random-init recipe (std 0.02, per-sublayer log-uniform [1e-3,1] scales on W_o
 * and W_d, gains 1), bit-identical to the host generator for the same seed.
 * asd_load_weights_file reads a flat file: 8 bytes "ASDW0001", int32[8] =
 * {n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab, dtype}, then
 * EMBED, FINAL_NORM, LM_HEAD, then per layer ATTN_NORM, WQ, WK, WV, WO, MLP_NORM,
 * WG, WU, WD, each as asd_set_weight takes it.
 */
int asd_set_weight(asd_engine* e, int32_t tensor_id, int32_t layer, const void* src, size_t bytes, int32_t src_on_device);
int asd_get_weight(asd_engine* e, int32_t tensor_id, int32_t layer, void* dst, size_t bytes);
int asd_init_synthetic(asd_engine* e, uint64_t seed);
int asd_load_weights_file(asd_engine* e, const char* path);

/*
 * Paged KV cache.  Logical page i (tokens [i*page_tokens, (i+1)*page_tokens)) lives
 * in physical page table[i]; table must be a permutation of 0..n_pages-1 where
 * n_pages = ceil(max_seq / page_tokens).  Default: identity.  Requires kv_len == 0.
 */
int asd_set_page_table(asd_engine* e, const int32_t* table, int32_t n_pages);

/*
 * The cache rows of positions pos0 .. pos0 + n - 1 of one layer, as the decode attention reads them (Section 1: the
 * cache a decoded token reloads): k_out and v_out are HOST arrays [n][n_kv_heads][head_dim] of fp32 (the stored
 * values widened; K after the rotary embedding), looked up through the page table.  Any position below the cache
 * capacity may be read, also beyond the current length (a never-written slot reads as 0, a slot left by a rejected
 * draft holds that draft's values).  Synchronises the stream.  Either output may be NULL.
 */
int asd_get_kv(asd_engine* e, int32_t layer, int32_t pos0, int32_t n, float* k_out, float* v_out);

/* Cache length control: reset = truncate to 0; truncate rolls back to new_len <= kv_len. */
int asd_reset(asd_engine* e);
int asd_truncate(asd_engine* e, int32_t new_len);
int32_t asd_kv_len(const asd_engine* e);

/*
 * Forward pass with an explicit skip mask (the draft model is the full model minus
 * the masked sublayers; NULL mask = full model).  tokens[n_rows] are fed at
 * positions pos0 .. pos0+n_rows-1; pos0 must equal asd_kv_len() (ASD_E_STATE
 * otherwise) and 1 <= n_rows <= max_rows.  commit != 0 leaves kv_len at
 * pos0+n_rows, else at pos0.  Outputs, each optional (NULL):
 *   logits [n_rows][vocab] fp32; cos [2L] = mean over the rows of the per-row
 *   cosine similarity of every sublayer (a removed sublayer reports exactly 1);
 *   cos_rows [n_rows][2L]; argmax [n_rows] (lowest index on ties).
 */
int asd_forward(asd_engine* e, const int32_t* tokens, int32_t n_rows, int32_t pos0, const uint8_t* skip_mask,
                int32_t commit, float* logits, float* cos, float* cos_rows, int32_t* argmax);

/*
 * asd_forward for callers that cannot allocate device memory or wait for the device while they enqueue work: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same pass, same kernels, same
 * bits as asd_forward, but
 *   - d_tokens [n_rows] is a DEVICE pointer, and so are the outputs d_logits [n_rows][vocab], d_cos [2L] (mean over
 *     the rows; a removed sublayer reports exactly 1) and d_argmax [n_rows], each optional (NULL); skip_mask is a
 *     HOST array, read before the call returns;
 *   - everything is enqueued on the engine's stream and the call returns without synchronising: the outputs are
 *     valid once the stream has reached this point;
 *   - the kernels' scratch (partial sums of the cosine taps and norms, attention partials and their arrival counters,
 *     argmax candidates) lives in a static device array of the library, ASD_NOALLOC_SCRATCH_BYTES per GPU, held until
 *     the process ends, instead of in the engine's arena.  The call allocates nothing on the device and calls no
 *     allocating runtime routine.  A pass whose scratch does not fit (it grows with heads x head_dim x context:
 *     the 7B shape fits up to 7680 positions) is refused with ASD_E_NOMEM;
 *   - every such call on a GPU uses that GPU's one array: calls that overlap on one GPU (two engines, two streams)
 *     race.  The array keeps the last call's contents; the call clears what must start at zero itself;
 *   - a token id outside the vocabulary cannot be refused up front (the ids are on the device): it is replaced by
 *     token 0 and raises a device flag that asd_check reports.
 * pos0 must equal asd_kv_len(); commit != 0 leaves kv_len at pos0 + n_rows.
 * asd_check synchronises the engine's stream and returns ASD_OK, or the error a kernel flagged since the last pass
 * started (ASD_E_INVAL: token id outside the vocabulary; ASD_E_STATE: a row of logits without a finite maximum).
 */
#define ASD_NOALLOC_SCRATCH_BYTES (8u << 20)
int asd_forward_noalloc(asd_engine* e, const int32_t* d_tokens, int32_t n_rows, int32_t pos0, const uint8_t* skip_mask,
                        int32_t commit, float* d_logits, float* d_cos, int32_t* d_argmax);
int asd_check(asd_engine* e);

/*
 * Prompt pass (Section 3.2, the definition of C_l): resets the cache, runs all n prompt tokens
 * through the full model, returns the first generated token, the ACS of every
 * sublayer over the n rows (cos_out [2L], optional) and the logits of the last row
 * (last_logits [vocab], optional).  The ACS is kept in the engine for a following
 * asd_decode with mask_mode 0.  Prompts longer than max_rows are processed in blocks
 * of up to 512 rows, layer by layer, with large-M matrix-core contractions (every
 * weight is read once per block); shorter ones as one pass of the decode kernels.
 * asd_prefill_chunked always takes the decode kernels, max_rows rows at a time (the
 * same results up to rounding; kept for cross-checks and as the reference for timing).
 * All pointers are host memory.
 */
int asd_prefill(asd_engine* e, const int32_t* tokens, int32_t n, int32_t* first_token, float* cos_out, float* last_logits);
int asd_prefill_chunked(asd_engine* e, const int32_t* tokens, int32_t n, int32_t* first_token, float* cos_out, float* last_logits);

/*
 * Algorithm 1 (ADMG), a pure host function: c_attn [L] are the attention sublayers'
 * ACS values; skip_mask [2L] receives remove_ATTN (even indices) and remove_MLP
 * (odd indices).  Layer l (0-based) is the paper's layer l+1: rule 1 removes it when
 * (l+1) % m == 0, rule 2 protects l >= L-n, CS thresholding removes attention l
 * when c_attn[l] >= alpha (compared in fp32).
 */
int asd_admg(const float* c_attn, int32_t n_layers, float alpha, int32_t m, int32_t n, int32_t use_cs, uint8_t* skip_mask);

/*
 * Algorithm 1 plus CS thresholding of the MLP sublayers (an extension): c_all [2L] holds
 * every sublayer's ACS (attention at even, MLP at odd indices); MLP l is also removed when
 * use_cs_mlp != 0, c_all[2l+1] >= alpha_mlp and rule 2 does not protect it.  With
 * use_cs_mlp == 0 the result equals asd_admg on the attention half.  Host function.
 */
int asd_admg2(const float* c_all, int32_t n_layers, float alpha, int32_t m, int32_t n, int32_t use_cs, float alpha_mlp,
              int32_t use_cs_mlp, uint8_t* skip_mask);

/*
 * Greedy speculative decoding from the current cache state (Section 1): last_token
 * is the newest token, not yet in the cache.  Emits exactly n_more tokens into
 * out_tokens; they equal what plain greedy decoding of the full model emits.  Each
 * cycle drafts min(k, tokens still needed - 1) tokens with the masked model,
 * verifies them in one pass of the full model, keeps the accepted prefix plus the
 * full model's token after it, and rolls the cache back to the accepted length.
 * mask_used [2L] (optional) receives the skip mask in effect.
 */
int asd_decode(asd_engine* e, int32_t last_token, int32_t n_more, const asd_gen_params* p,
               int32_t* out_tokens, asd_gen_stats* stats, uint8_t* mask_used);

/*
 * The sampling kernels on caller-given logits (host arrays): q_logits [kk][vocab] are draft-model
 * logits, p_logits [kk+1][vocab] the full model's for the same positions plus the next.  Draws the
 * kk draft tokens (drafts_out [kk], output indices index0 .. index0+kk-1), verifies them by
 * speculative sampling and returns the number kept (*n_accepted) and the token that follows them
 * (*next_token).  0 <= kk < max_rows, temperature > 0.  Does not touch the KV cache.  For callers
 * that bring their own logits, and for checking the kernels against the rule on known inputs.
 */
int asd_spec_sample(asd_engine* e, const float* q_logits, const float* p_logits, int32_t kk, float temperature, uint64_t seed,
                    int64_t index0, int32_t* drafts_out, int32_t* n_accepted, int32_t* next_token);

/* asd_prefill + ADMG + asd_decode: out_tokens [n_new], out_tokens[0] is the prompt pass's token. */
int asd_generate(asd_engine* e, const int32_t* prompt, int32_t n_prompt, int32_t n_new, const asd_gen_params* p,
                 int32_t* out_tokens, asd_gen_stats* stats, uint8_t* mask_used);

/* Per-kernel-class GPU time of one profiled prompt pass in blocks (asd_prefill's path for prompts of more than
 * max_rows tokens); flops = multiply-adds x 2 of the class's contractions, each counted once. */
enum { ASD_PK_ROWS = 0, ASD_PK_QKV = 1, ASD_PK_ATTN = 2, ASD_PK_OPROJ = 3, ASD_PK_GATEUP = 4, ASD_PK_DOWN = 5,
       ASD_PK_LMHEAD = 6, ASD_PK_COUNT = 7 };
typedef struct {
    double ms[ASD_PK_COUNT];
    int32_t launches[ASD_PK_COUNT];
    double flops[ASD_PK_COUNT];
    double ms_total;
} asd_prefill_times;

/*
 * Measurement helpers (benchmark only; they leave kv_len unchanged, except asd_profile_prefill).
 * asd_time_pass: average milliseconds of one forward pass of n_rows rows at the
 * current kv_len with the given mask, over reps back-to-back repetitions bracketed
 * by HIP events on the engine's stream (as a captured graph when use_graph != 0);
 * *bytes (optional) = algorithmic bytes one such pass must read.
 * asd_profile_forward: one such pass with an event pair around every launch.
 * asd_time_step_class: the steps of one kernel class (ASD_K_QKV .. ASD_K_LMHEAD, one per kept layer) of a full-model
 * pass launched back to back, reps rounds, bracketed by one pair of HIP events on the engine's stream: average
 * microseconds per launch (weights differ from launch to launch, so no launch finds its weights cached) and the
 * algorithmic bytes one launch must read.  The steps run out of their usual order: the pass's activations are
 * scratch afterwards.
 * asd_profile_prefill: the prompt pass in blocks over n > max_rows tokens (host array), once untimed and once with
 * an event pair around every launch; ASD_PK_ROWS collects the row-wise kernels (embedding, residual add + cosine
 * tap), ASD_PK_LMHEAD the last row's hand-over, LM head and argmax.  Resets the cache (kv_len 0 afterwards).
 * asd_copy_bench: average milliseconds of a plain device copy kernel moving
 * nbytes (read nbytes + write nbytes) inside the arena's scratch region; used to
 * calibrate byte counters and to report the achievable HBM rate.
 */
int asd_time_pass(asd_engine* e, int32_t n_rows, const uint8_t* skip_mask, int32_t reps, int32_t use_graph,
                  double* ms_avg, double* bytes);
int asd_profile_forward(asd_engine* e, int32_t n_rows, const uint8_t* skip_mask, asd_kernel_times* out);
int asd_time_step_class(asd_engine* e, int32_t cls, int32_t n_rows, int32_t reps, double* us_avg, double* bytes_per_launch);
int asd_profile_prefill(asd_engine* e, const int32_t* tokens, int32_t n, asd_prefill_times* out);
int asd_copy_bench(asd_engine* e, size_t nbytes, int32_t reps, double* ms_avg);

#ifdef __cplusplus
}
#endif
#endif /* ASD_H */
