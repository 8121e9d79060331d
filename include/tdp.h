/*
 * tdp.h - C ABI of the MI355X pipeline-stage library.
 *
 * One "stage" is a contiguous slice of a Llama-style model's decoder layers held by one GPU
 * (paper Sec. 2.2.3: pipeline parallelism splits the model layer-wise, each device owning a
 * subset of layers).  A stage is told which batch to run and in which phase (Sec. 3.2: the
 * engine packs prompts for the prefill phase and decode steps for the decode phase; a worker
 * only knows what to compute); batches are never mixed (separate batching, Sec. 2.3, Sec. 3.1).
 * Hidden states come in from the previous stage and go out to the next: no embedding, no final
 * norm, no LM head.
 *
 * Conventions
 *  - All functions return TDP_OK (0) or a negative error code; tdp_last_error() gives a
 *    thread-local message for the most recent failure.
 *  - Argument checks run on the host before any GPU work, so a bad argument never launches.
 *  - "dev" pointers are device (HBM) addresses, "host" pointers are ordinary host addresses.
 *  - bf16 is the raw 16-bit brain-float encoding; matrices are row-major.
 *  - Calls that take a `stream` (a hipStream_t passed as void*, NULL = the default stream) only
 *    enqueue work and return; nothing synchronises with the host.  One stage must not be driven
 *    from two streams at once: its scratch buffers are shared.
 *  - The caller owns page allocation: which physical page belongs to which request is the
 *    engine's business (Sec. 3.2.1).  The stage only writes the slot the tables name.
 *    Contents of device-side tables are trusted by the prefill / decode / import / export calls:
 *    a page id outside [0, num_pages) or a position beyond 16 * max_pages_per_seq is undefined
 *    behaviour there.  tdp_stage_check_decode / tdp_stage_check_prefill validate them first for a
 *    caller that wants that (they cost a synchronisation, so they are not part of the hot calls).
 */
#ifndef TDP_H_
#define TDP_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TDP_API __attribute__((visibility("default")))

#define TDP_OK       0
#define TDP_EINVAL  (-1)   /* null pointer, bad shape, size beyond the configured maximum */
#define TDP_ENOMEM  (-2)   /* device or host allocation failed */
#define TDP_EHIP    (-3)   /* a HIP runtime call failed (message holds the HIP error string) */

/* weight identifiers for tdp_stage_set_weight */
#define TDP_WQ      0      /* [d_model, n_q_heads*head_dim]  */
#define TDP_WK      1      /* [d_model, n_kv_heads*head_dim] */
#define TDP_WV      2      /* [d_model, n_kv_heads*head_dim] */
#define TDP_WO      3      /* [n_q_heads*head_dim, d_model]  */
#define TDP_WG      4      /* [d_model, d_ff]   gate         */
#define TDP_WU      5      /* [d_model, d_ff]   up           */
#define TDP_WD      6      /* [d_ff, d_model]   down         */
#define TDP_G_ATTN  7      /* [d_model] RMSNorm gain before attention */
#define TDP_G_MLP   8      /* [d_model] RMSNorm gain before the MLP   */
/* optional biases of the q / k / v projections (the Qwen2.5-32B model of the paper's Table 2 has
 * them; a stage whose biases are never set runs without): vectors [d_q, 1], [d_kv, 1], [d_kv, 1] */
#define TDP_BQ 9
#define TDP_BK 10
#define TDP_BV 11

#define TDP_F32     0
#define TDP_BF16    1

#define TDP_HOST    0
#define TDP_DEVICE  1

/* element type of the KV pools (tdp_stage_config.kv_dtype) */
#define TDP_KV_BF16      0
#define TDP_KV_FP8_E4M3  1   /* OCP 8-bit float, 4 exponent bits (bias 7), 3 mantissa bits, max 448, no infinities */

typedef struct tdp_stage tdp_stage;   /* opaque: owns weights, KV pools and scratch (all in HBM) */

typedef struct tdp_stage_config {
  int32_t n_layers;            /* decoder layers in this stage (>= 1) */
  int32_t d_model;             /* multiple of 64 */
  int32_t n_q_heads;           /* multiple of n_kv_heads; group size n_q_heads/n_kv_heads <= 16 */
  int32_t n_kv_heads;
  int32_t head_dim;            /* 64 or 128 */
  int32_t d_ff;                /* SwiGLU width, multiple of 4 */
  float   rms_eps;
  float   rope_base;
  int32_t page_size;           /* tokens per KV page; must be 16 */
  int32_t num_pages;           /* physical pages per layer in the KV pool */
  int32_t max_batch;           /* largest decode batch */
  int32_t max_tokens;          /* largest packed prefill token count */
  int32_t max_seqs;            /* largest number of prompts in one prefill */
  int32_t max_pages_per_seq;   /* width of a block-table row */
  /* KV-cache element type.  The decode phase is bound by reading the cache (Sec. 2.1); the paper keeps
   * it in the model's 16-bit type (TDP_KV_BF16, the default and what every headline number uses).
   * TDP_KV_FP8_E4M3 stores each key (after rotation) and value as the E4M3 code of value / scale:
   * round to nearest, ties to the even code, magnitudes from 448 up saturate, NaN stays NaN; the
   * quotient is an fp32 division.  Attention in both phases reads the cache, i.e. code * scale (the
   * code value is exact in bf16; the scales join the softmax scale and the final normalisation), and
   * is otherwise unchanged.  k_scale / v_scale: per stage, > 0; 0 means 1. */
  int32_t kv_dtype;
  float   k_scale, v_scale;
  /* Decode batches as two half-batches on two streams (0 or 1: off, the default; 2: on).  The decode
   * phase alternates a step bound by reading the cache (attention) with steps bound by the matrix
   * cores (the projections, Sec. 2.1 and Sec. 3.4); with two half-batches in flight one half's attention
   * may run beside the other half's projections.  The stage then holds a second set of scratch buffers
   * and a second stream of its own (default priority); tdp_stage_decode forks it behind the work already
   * queued on the caller's stream and joins it before returning control of that stream, so callers see
   * the same semantics (graph capture included).  Results equal the one-batch form's within rounding;
   * per-class timing is not recorded in this form.  Measured slower than one batch on MI355X at the
   * benchmark shapes (each half streams all weights again): an option, not the default. */
  int32_t decode_micro_batches;
} tdp_stage_config;

/* Version of this ABI (bumped on incompatible change). */
TDP_API int tdp_abi_version(void);

/* Message for the calling thread's most recent error ("" if none).  Never NULL. */
TDP_API const char* tdp_last_error(void);

/*
 * Create a stage: allocates weights (zeroed), per-layer K and V pools and scratch on the current
 * HIP device.  `*out` is set only on success.  Errors: TDP_EINVAL (bad config), TDP_ENOMEM,
 * TDP_EHIP.  The config is checked before any HIP call.
 */
TDP_API int tdp_stage_create(const tdp_stage_config* cfg, tdp_stage** out);

/* Free everything the stage owns.  NULL is allowed.  Synchronises the device first. */
TDP_API void tdp_stage_destroy(tdp_stage* st);

/*
 * Load one weight.  `src` is a row-major [rows, cols] = [in, out] matrix (y = x W) or a vector
 * [rows] with cols = 1, of type `dtype` (TDP_F32 or TDP_BF16; fp32 is rounded to bf16 with
 * round-to-nearest-even, gains are kept in fp32), living where `mem` says (TDP_HOST or
 * TDP_DEVICE).  The library repacks it once into its own MFMA-friendly layout; `src` is not
 * referenced after the call returns (the call synchronises).  Shapes must match the config.
 */
TDP_API int tdp_stage_set_weight(tdp_stage* st, int32_t layer, int32_t which, const void* src,
                         int32_t dtype, int32_t mem, int64_t rows, int64_t cols);

/*
 * Raw access to one layer's KV pools, for tests that poison, inject or dump them.
 * Layout:  K pool [num_pages][n_kv_heads][R / 64][16][64 bytes]   (R = bytes of one key row)
 *          V pool [num_pages][n_kv_heads][head_dim][16]             (token slot fastest)
 * of bf16 elements, or of one-byte E4M3 codes when kv_dtype = TDP_KV_FP8_E4M3.  A key row (head_dim
 * elements, R = 64 ... 256 bytes) is stored in 64-byte pieces, piece g of the page's 16 token slots
 * together: byte r of the key of (page, head, slot) lies at
 *   ((page * n_kv_heads + head) * 16 * R) + (r / 64) * 1024 + slot * 64 + r % 64
 * (what one decode-attention load instruction fetches, 64 bytes of each of 16 tokens, is then four
 * runs of 256 bytes instead of sixteen half cache lines).
 * Keys are stored after the rotary embedding.  `*bytes` = size of EACH pool.
 */
TDP_API int tdp_stage_kv_pool(tdp_stage* st, int32_t layer, void** k_dev, void** v_dev, int64_t* bytes);

/*
 * Copy K/V between packed logical order and the pages (the path a recompute-free migration or a
 * test would use).  k_packed / v_packed: dev bf16 [total_tokens][n_kv_heads][head_dim], the
 * sequences' tokens concatenated; token t of sequence s (cu_seqlens[s] <= t < cu_seqlens[s+1])
 * lives at position t - cu_seqlens[s], i.e. page block_tables[s][pos/16], slot pos%16.
 * cu_seqlens: dev int32 [n_seqs+1]; block_tables: dev int32 [n_seqs][max_pages_per_seq].
 * import writes pages from the packed arrays, export reads pages into them.  With an 8-bit cache
 * the packed side stays bf16: import stores the code of value / scale, export returns
 * bf16(code * scale).
 */
TDP_API int tdp_stage_kv_import(tdp_stage* st, int32_t layer, const void* k_packed, const void* v_packed,
                        const int32_t* cu_seqlens, const int32_t* block_tables, int32_t n_seqs,
                        int32_t total_tokens, void* stream);
TDP_API int tdp_stage_kv_export(tdp_stage* st, int32_t layer, void* k_packed, void* v_packed,
                        const int32_t* cu_seqlens, const int32_t* block_tables, int32_t n_seqs,
                        int32_t total_tokens, void* stream);

/*
 * Prefill phase (Sec. 2.1: all prompt tokens are processed concurrently and the KV cache is
 * initialised).  Runs every layer of the stage over `total_tokens` packed prompt tokens.
 *   hidden_in    dev bf16 [total_tokens][d_model]   packed var-length prompts
 *   cu_seqlens   dev int32 [n_seqs+1]               prefix sums of prompt lengths, [0] = 0
 *   block_tables dev int32 [n_seqs][max_pages_per_seq]; row s needs ceil(len_s/16) valid entries
 *   hidden_out   dev bf16 [total_tokens][d_model]   (may alias hidden_in)
 * Every prompt starts at position 0 on an empty cache (no chunked prefill, Sec. 2.3); attention
 * is causal within a prompt; K (rotated) and V of every token and layer are written to the
 * pages.  n_seqs <= max_seqs, total_tokens <= max_tokens, each prompt <= 16*max_pages_per_seq.
 * n_seqs = 0 or total_tokens = 0 is a successful no-op.
 */
TDP_API int tdp_stage_prefill(tdp_stage* st, const void* hidden_in, const int32_t* cu_seqlens,
                      const int32_t* block_tables, int32_t n_seqs, int32_t total_tokens,
                      void* hidden_out, void* stream);

/*
 * Decode phase (Sec. 2.1: each step processes one new token per request using the KV cache).
 *   hidden_in    dev bf16 [batch][d_model]          one token per request
 *   ctx_lens     dev int32 [batch]                  tokens ALREADY cached for request b; the new
 *                                                   token takes position ctx_lens[b]
 *   block_tables dev int32 [batch][max_pages_per_seq]; row b needs ceil((ctx_lens[b]+1)/16) entries
 *   hidden_out   dev bf16 [batch][d_model]          (may alias hidden_in)
 * For every layer the new token's K (rotated) and V are appended at page
 * block_tables[b][ctx/16], slot ctx%16 BEFORE attention, which then spans ctx+1 tokens.
 * ctx_lens[b] = 0 is legal.  batch <= max_batch; batch = 0 is a successful no-op.  Re-running a
 * step with the same inputs rewrites the same slots with the same values.
 */
TDP_API int tdp_stage_decode(tdp_stage* st, const void* hidden_in, const int32_t* ctx_lens,
                     const int32_t* block_tables, int32_t batch, void* hidden_out, void* stream);

/*
 * Validate the device-side tables of a decode or prefill call before making it.  Checked, for every
 * row of the batch: the length (decode: 0 <= ctx_lens[b] and ctx_lens[b] + 1 <= 16 * max_pages_per_seq;
 * prefill: 0 <= len_s <= 16 * max_pages_per_seq, cu_seqlens[0] = 0, cu_seqlens[n_seqs] = total_tokens);
 * every table entry the call would use lies in [0, num_pages); and no page that the call writes
 * (decode: the page of position ctx_lens[b]; prefill: every page of every prompt) appears a second
 * time among the entries the call uses - two requests writing one page, or one reading what another
 * writes, is how a page-allocation mistake shows (the engine owns allocation, Sec. 3.2.1).  Pages
 * that are only read may be shared.  The kernels read the tables inside [rows][max_pages_per_seq]
 * whatever the lengths say, so the check itself is safe on arbitrary input.
 * Returns TDP_OK, or TDP_EINVAL with a message naming the first offending row and what is wrong
 * with it.  Same size limits and pointer kinds as the call it guards.  Runs on `stream` and waits for it.
 */
TDP_API int tdp_stage_check_decode(tdp_stage* st, const int32_t* ctx_lens, const int32_t* block_tables,
                                   int32_t batch, void* stream);
TDP_API int tdp_stage_check_prefill(tdp_stage* st, const int32_t* cu_seqlens, const int32_t* block_tables,
                                    int32_t n_seqs, int32_t total_tokens, void* stream);

/*
 * Restrict the following prefill/decode calls to layers [first, first + count) of the stage, as
 * if the stage were that sub-slice (a finer pipeline split, or a layer-by-layer check against a
 * reference).  The hand-over format at both ends stays bf16.  count = 0 restores the whole stage.
 * Errors: TDP_EINVAL when the range does not lie inside [0, n_layers).
 */
TDP_API int tdp_stage_set_layer_range(tdp_stage* st, int32_t first, int32_t count);

/*
 * Decode attention splits a request's context into spans of `span_tokens` logical tokens, one
 * workgroup per (span, K/V head), and merges the spans' partial softmax states in a fixed logical
 * order (Sec. 2.1: a decode step reads the request's whole cache).  By default the span is chosen
 * from batch x K/V heads so that small batches still fill the GPU; this call pins it for the
 * following decode calls (tuning, and tests that walk every span length).  span_tokens: 0 =
 * automatic, else 256, 512, 1024, 2048 or 4096.  Results agree within rounding whatever the span.
 */
TDP_API int tdp_stage_set_decode_span(tdp_stage* st, int32_t span_tokens);

/*
 * Diagnostic: one projection GEMM through the library's kernels, out = A * W with W given as
 * a row-major [K, N] bf16 device matrix (repacked internally on every call: not a fast path).
 * A dev bf16 [M][K]; out dev bf16 [M][N].  K multiple of 64, N multiple of 4.
 * tile: 0 = automatic, 1..3 force a kernel variant (256 x 256, 128 x 256, 128 x 128 output tile);
 * splits: 0 = automatic, else force the split-K factor.  epilogue: 0 = plain store; 1 = out =
 * residual + A*W (residual dev bf16 [M][N]); 2 = the gated MLP epilogue (Sec. 3.4 counts the MLP among
 * the linear layers that dominate a decode step): W = [W_gate | W_up] side by side, N = 2 F, and
 * out dev bf16 [M][F] = silu(A*W_gate) * (A*W_up) with silu(z) = z / (1 + exp(-z)); F multiple of 4.
 */
TDP_API int tdp_gemm_bf16(const void* A, const void* W, const void* residual, void* out, int32_t M, int32_t N,
                  int32_t K, int32_t epilogue, int32_t tile, int32_t splits, void* stream);

/*
 * tdp_gemm_bf16 (epilogues 0 and 1) for callers that cannot allocate device memory (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): same kernels, same results, but
 * the repacked weights and the split-K partials live in a device array that is part of the library
 * image (64 MiB per GPU, held until the process ends) instead of two allocations per call.  The
 * call allocates and frees nothing and only enqueues on `stream` (it does not wait; the caller
 * synchronises before reading `out`).  Limits: N rounded up to a multiple of 256, times K, at most
 * 8 Mi elements (16 MiB of weights); (splits, or 16 when splits = 0) * M * that N at most 12 Mi
 * floats (48 MiB of partials); anything larger is TDP_EINVAL with a message naming the limit, checked
 * before any GPU work.  All calls on one GPU share the one array: calls that may overlap (different
 * streams without an order between them, or several threads) race; calls on one stream are safe.
 */
TDP_API int tdp_gemm_bf16_static(const void* A, const void* W, const void* residual, void* out, int32_t M,
                                 int32_t N, int32_t K, int32_t epilogue, int32_t tile, int32_t splits, void* stream);

/*
 * Diagnostics for the 8-bit cache format: the conversions exactly as the KV kernels perform them.
 * tdp_e4m3_from_f32: codes[i] = E4M3 code of src[i] / scale (dev fp32 -> dev bytes; scale > 0).
 * tdp_e4m3_to_f32:   dst[i] = value of codes[i] (dev bytes -> dev fp32), through the conversion
 *                    instruction the decode-attention kernel uses; n a multiple of 4, codes 4-byte
 *                    and dst 16-byte aligned.
 */
TDP_API int tdp_e4m3_from_f32(const float* src, uint8_t* codes, int64_t n, float scale, void* stream);
TDP_API int tdp_e4m3_to_f32(const uint8_t* codes, float* dst, int64_t n, void* stream);

/*
 * Empirical ceilings of the GPU the library runs on, for the benchmark's roofline context (the
 * decode phase is bound by memory bandwidth and the prefill phase by compute, Sec. 2.1; these say
 * what the part sustains for either with no other work in the way).  Both calls launch a trivial
 * kernel `launches` times (1..1000) after one warm-up, time the launches with HIP events on
 * `stream`, wait for them and return the average milliseconds per launch in *ms_per_launch (host).
 * tdp_probe_hbm_read: reads the first 2^k * 4 KiB of `buf` (dev, 16-byte aligned, at least 512 KiB;
 *   2^k * 4 KiB is the largest such size <= bytes, returned in *bytes_per_launch) exactly once per
 *   launch, 16 bytes per lane per instruction, 16 KiB in flight per wave.  pattern bit 0: 0 walks the
 *   4 KiB pieces in address order, 1 in a fixed pseudo-random order (how a paged KV cache is read);
 *   bit 1: the loads are marked non-temporal, as the library's own kernels mark data they read once
 *   (keys and values in decode, weights of a GEMM with a single row of tiles).  Nothing is written to `buf`.
 * tdp_probe_mfma_bf16: `iters` (1..2^22) rounds of sixteen independent 16x16x32 bf16 MFMAs per wave on
 *   register operands, two waves per SIMD on every CU; *flop_per_launch (host) = multiply-adds * 2.
 *   random_operands = 1: operands uniform in (-1, 1), different in every lane and element; 0: the
 *   same constants everywhere (the rate depends on it: the part is power-limited and an MFMA's
 *   power grows with the operand bits that toggle).
 * Errors: TDP_EINVAL (null pointer, size or count out of range), TDP_ENOMEM, TDP_EHIP.
 */
TDP_API int tdp_probe_hbm_read(const void* buf, int64_t bytes, int32_t pattern, int32_t launches,
                               int64_t* bytes_per_launch, float* ms_per_launch, void* stream);
TDP_API int tdp_probe_mfma_bf16(int32_t iters, int32_t launches, int32_t random_operands, double* flop_per_launch,
                                float* ms_per_launch, void* stream);

/*
 * Timing hooks: when enabled, prefill/decode record HIP events around each kernel class on the
 * call's stream; tdp_stage_timing_read synchronises and returns the summed milliseconds of the
 * most recent call per class (order: rmsnorm, gemm_qkv, rope_kv, attention, gemm_o, gemm_gate_up,
 * gemm_down, attention_merge) into ms[8].  "attention" is the attention kernel alone (prefill or
 * decode), "attention_merge" the kernel that combines the partial results of decode requests longer
 * than one span (0 in prefill, and when no request of the batch can be that long).
 */
TDP_API int tdp_stage_timing_enable(tdp_stage* st, int32_t on);
TDP_API int tdp_stage_timing_read(tdp_stage* st, float* ms /* host [8] */);

/* ---- the two ends of the pipeline ---------------------------------------------------------------
 * What runs in front of the first stage and behind the last one so that a chain of stages turns
 * token ids into token ids (the paper measures generated tokens per second on whole models, Sec.
 * 4.1 and Table 2): the token-embedding lookup, and the final RMSNorm + vocabulary projection +
 * greedy selection.  A tdp_ends owns the embedding table (bf16 [vocab, d_model]), the final norm
 * gain (fp32) and the vocabulary projection (bf16, repacked once), plus scratch for max_tokens rows.
 * vocab_size must be a multiple of 4, d_model a multiple of 64. */
typedef struct tdp_ends tdp_ends;
typedef struct {
  int32_t vocab_size, d_model;
  float rms_eps;
  int32_t max_tokens; /* rows per call */
} tdp_ends_config;
#define TDP_E_EMBEDDING 0  /* [vocab_size, d_model] */
#define TDP_E_FINAL_NORM 1 /* [d_model, 1] */
#define TDP_E_LM_HEAD 2    /* [d_model, vocab_size] row-major ([in, out] like every projection) */
TDP_API int tdp_ends_create(const tdp_ends_config* cfg, tdp_ends** out);
TDP_API void tdp_ends_destroy(tdp_ends* e);
/* src: host or device (mem), fp32 or bf16 (dtype); synchronous */
TDP_API int tdp_ends_set_weight(tdp_ends* e, int32_t which, const void* src, int32_t dtype, int32_t mem,
                                int64_t rows, int64_t cols);
/* hidden_out[m][:] = embedding[token_ids[m]][:].  token_ids dev int32 [M]; hidden_out dev bf16
 * [M, d_model].  An id outside the vocabulary is clamped into it (never a wild read).  Enqueues on
 * stream and returns. */
TDP_API int tdp_embed_tokens(tdp_ends* e, const int32_t* token_ids, int32_t M, void* hidden_out, void* stream);
/* For row m: x = hidden_in[row_index ? row_index[m] : m]; logits[m] = RMSNorm(x; gain) * W_head;
 * next_token[m] = the lowest index among the largest logits.  hidden_in dev bf16 [n_rows_in,
 * d_model]; row_index dev int32 [M] or null (prefill: the last token of each prompt), entries are
 * clamped to [0, n_rows_in); logits_out dev fp32 [M, vocab_size] or null (internal scratch);
 * next_token dev int32 [M] or null.  M <= max_tokens.  fp32 accumulation, fp32 logits. */
TDP_API int tdp_lm_head(tdp_ends* e, const void* hidden_in, int32_t n_rows_in, const int32_t* row_index, int32_t M,
                        float* logits_out, int32_t* next_token, void* stream);
/* Greedy selection alone: out[m] = lowest index among the maxima of logits[m][0..n), rows ld apart.
 * All device pointers.  NaN entries never win; a row of NaNs gives 0. */
TDP_API int tdp_argmax_rows(const float* logits, int32_t M, int32_t n, int64_t ld, int32_t* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TDP_H_ */
