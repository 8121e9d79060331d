// Host-side launch interface of the HIP kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tdp {

// ---- operand layouts -----------------------------------------------------------------------------
// Element (row r, column k) of a GEMM operand lives at
//     (r >> shift) * group + (k >> 5) * kb + (r & (2^shift - 1)) * par + (k & 31)
// i.e. rows are taken in groups of 2^shift, and inside a group the rows alternate in 32-column
// blocks, so one 32-wide k step of a whole group is one contiguous piece of 2^shift * 64 bytes.
// Row-major with leading dimension ld:  shift 1, group = 2 ld, kb = 32, par = ld.
// Pair-interleaved (groups of 2: a 128-byte line per k step): shift 1, group = 2 K, kb = 64, par = 32;
// the layout of the activations the stage's own kernels hand to the GEMMs, which lets a k-stage of 32
// be fetched with full-line requests.
// Blocked (groups of R = 2^shift rows, R * 64 contiguous bytes per k step): group = R K, kb = 32 R,
// par = 32; the layout of the repacked weights, R = 128: a direct-to-LDS instruction (16 rows x 64
// bytes) then covers one contiguous KiB, and a workgroup that streams its rows over k reads HBM in
// 8 KiB pieces (measured on a 57344 x 8192 matrix: 6.0-6.2 TB/s with groups of 64 or 128 against
// 5.3-5.5 with groups of 2; in the stage, groups of 128 are 1-2 % ahead of 64 and of 256).
struct OperandLayout {
  int64_t group, kb, par;
  int shift;
};
static inline OperandLayout layout_row_major(int64_t ld) { return OperandLayout{2 * ld, 32, ld, 1}; }
static inline OperandLayout layout_paired(int64_t K) { return OperandLayout{2 * K, 64, 32, 1}; }
constexpr int kWeightGroupShift = 7;  // weights: groups of 128 rows
static inline OperandLayout layout_weights(int64_t K) {
  return OperandLayout{(int64_t)(1 << kWeightGroupShift) * K, 32ll << kWeightGroupShift, 32, kWeightGroupShift};
}

// ---- GEMM: out[M, N] = epilogue(A[M, K] * W^T), W stored [Npad][Kpad] (K contiguous) ---------
enum Epilogue : int {
  EPI_STORE = 0,     // out = acc                        (QKV projection)
  EPI_RESIDUAL = 1,  // out = residual + acc             (O and down projections)
  EPI_SWIGLU = 2,    // out[:, j] = silu(gate_j) * up_j  (gate/up projection; W rows interleaved
                     //                                   in blocks of 32: gate block, up block)
};

constexpr int kGemmTileMax = 3;  // kernel variants: 1 = 256 x 256 tile, 2 = 128 x 256, 3 = 128 x 128
struct GemmArgs {
  const void* A;      // bf16, M rows x Kpad columns in a_layout; rows >= M are never read
  OperandLayout a_layout;
  const void* W;      // bf16, Npad rows x Kpad columns in layout_weights(Kpad), zero padded
  int64_t Kpad;       // multiple of 64
  int64_t Npad;       // multiple of 256
  int M;
  int N_store;        // columns of `out` that exist (SWIGLU: Npad/2 is stored up to N_store)
  void* out;          // [M][ldo], bf16 unless out_f32; EPI_SWIGLU: bf16 in u_layout instead
  int64_t ldo;
  OperandLayout u_layout;
  const float* bias;     // [Npad] fp32 or null: added to every row (plain / residual epilogues)
  const void* residual;  // [M][ldr] or null, bf16 unless residual_f32
  int64_t ldr;
  int epilogue;
  int out_f32;        // plain and residual epilogues: `out` is fp32 (residual stream inside a stage; logits)
  int residual_f32;
  float* workspace;       // fp32 split-K partials
  int64_t workspace_elems;
  int force_tile;         // 0 = choose; else 1..kGemmTileMax selects a kernel variant (tests / tuning)
  int force_splits;       // 0 = choose
  // Deferred reduction (plain and residual epilogues only): when the plan splits K, leave the fp32
  // partials in the workspace, ws[(z * M + m) * Npad + n] for split z, apply nothing and launch no
  // reduce kernel; *splits_used (host) receives the number of splits, 1 meaning `out` was written as
  // usual.  The consumer (launch_rmsnorm_sum, launch_rope_kv with partials) sums them.
  int* splits_used;       // null = reduce here
};
hipError_t launch_gemm(const GemmArgs& a, hipStream_t s);
hipError_t gemm_setup();  // one-time function attributes (dynamic LDS size)

// ---- weight repack: dst[row_of(n)][k] = src[k][n] -------------------------------------------
// mode 0: row_of(n) = row_off + n;  mode 1: gate rows  (n/32)*64 + n%32;  mode 2: up rows (+32)
// dst is in layout_weights(dst_ld)
hipError_t launch_repack(const void* src, int src_is_f32, int64_t rows_in /*K*/, int64_t cols_out /*N*/,
                         void* dst, int64_t dst_ld, int64_t row_off, int mode, hipStream_t s);
// the same from a source whose rows are ld_src elements apart (a column range of a wider matrix)
hipError_t launch_repack_ld(const void* src, int src_is_f32, int64_t rows_in, int64_t cols_out, int64_t ld_src,
                            void* dst, int64_t dst_ld, int64_t row_off, int mode, hipStream_t s);
hipError_t launch_convert_vec(const void* src, int src_is_f32, int64_t n, float* dst, hipStream_t s);

// ---- pipeline ends ----------------------------------------------------------------------------
// dst[m][:] = src[idx[m]][:] (bf16 rows of d elements, d a multiple of 8; indices clamped into range)
hipError_t launch_gather_rows(const void* src, int64_t ld_src, int64_t n_src_rows, const int32_t* idx, int M, int d,
                              void* dst, int64_t ld_dst, hipStream_t s);
hipError_t launch_to_bf16(const void* src, int src_is_f32, int64_t n, void* dst, hipStream_t s);
// out[m] = lowest index among the maxima of logits[m][0..n)
hipError_t launch_argmax_rows(const float* logits, int64_t ld, int M, int n, int32_t* out, hipStream_t s);

// ---- RMSNorm ---------------------------------------------------------------------------------
hipError_t launch_rmsnorm(const void* x, int x_is_f32, int64_t ldx, const float* gain, float eps, int M, int d,
                          void* y, OperandLayout y_layout, hipStream_t s);

// The same with the row formed on the fly from split-K partials: h[m] = residual[m] + sum_z ws[(z*M+m)*ld_ws + :],
// written to h_out (fp32, leading dimension ldh) and normalised into y.
hipError_t launch_rmsnorm_sum(const void* residual, int residual_is_f32, int64_t ldr, const float* ws, int splits,
                              int64_t ld_ws, float* h_out, int64_t ldh, const float* gain, float eps, int M, int d,
                              void* y, OperandLayout y_layout, hipStream_t s);

// ---- RoPE + KV append ------------------------------------------------------------------------
struct KvLayout {
  void* k_pool;   // [num_pages][Hkv][row bytes / 64][page = 16 tokens][64 bytes]   (see k_pool_byte)
  void* v_pool;   // [num_pages][Hkv][dh][page]   (token index fastest)
  int num_pages, n_kv_heads, head_dim, page_size;
  int fp8;        // 0: elements are bf16; 1: elements are E4M3 codes of value / scale (one byte each)
  float k_scale, v_scale;
};
// Byte offset into the K pool of byte `row_byte` of the key of (page, kv head, token slot).  A key row
// (head_dim elements: 256, 128 or 64 bytes) is cut into 64-byte pieces, and piece g of all 16 tokens
// of the page lies together (1 KiB).  The reason is the decode-attention load: one instruction fetches
// 64 bytes of each of 16 tokens (an MFMA operand is 16 rows x 32 k).  With whole rows contiguous those
// are sixteen half cache lines and the kernel streams 5.8 TB/s; piece-major they are four runs of
// 256 bytes and it streams what a plain copy does (6.9 TB/s; both measured with a load-only probe).
__host__ __device__ inline int64_t k_pool_byte(const KvLayout& kv, int64_t page, int kvh, int slot, int row_byte) {
  const int row_bytes = kv.head_dim * (kv.fp8 ? 1 : 2);
  return (page * kv.n_kv_heads + kvh) * (int64_t)(16 * row_bytes) + (row_byte >> 6) * 1024 + slot * 64 + (row_byte & 63);
}
// decode: token b sits at position ctx_lens[b] of sequence b.  prefill: token t of sequence s
// (cu_seqlens[s] <= t < cu_seqlens[s+1]) sits at position t - cu_seqlens[s].
// The projection is read in fp32: proj[(z * n_tokens + t) * ld + :] summed over the `splits` split-K
// partials z (splits = 1: the GEMM's finished fp32 output), plus `bias` if given.  The rotated
// queries are written to the bf16 rows qkv[t] (same ld), and so are the values in prefill.
hipError_t launch_rope_kv(void* qkv, int64_t ld, int n_tokens, int n_q_heads, const KvLayout& kv,
                          const float2* rope_table, int max_pos, const int32_t* ctx_lens,
                          const int32_t* cu_seqlens, int n_seqs, const int32_t* block_tables,
                          int max_pages_per_seq, const float* proj, int splits, const float* bias, hipStream_t s);
// KV import/export between packed logical order [tokens][Hkv][dh] and the paged pools.
hipError_t launch_kv_copy(int to_pages, void* k_packed, void* v_packed, const KvLayout& kv,
                          const int32_t* cu_seqlens, int n_seqs, int total_tokens,
                          const int32_t* block_tables, int max_pages_per_seq, hipStream_t s);

// Validation of the tables of a decode (lens = ctx_lens[n_rows]) or prefill (lens = cu_seqlens[n_rows + 1])
// call.  owner: scratch int32[num_pages]; res: int32[2] = {violations, min(row * 8 + kind)} with kind
// 1 = length, 2 = page id, 3 = written page shared, 4 = cu_seqlens ends.  Reads the tables in bounds on any input.
hipError_t launch_table_check(int decode, const int32_t* lens, const int32_t* tables, int n_rows,
                              int max_pages_per_seq, int num_pages, int total_tokens, int32_t* owner, int32_t* res,
                              hipStream_t s);

// ---- attention -------------------------------------------------------------------------------
// tokens of one request's context handled by one workgroup (multiples of 128: four waves, 32-token blocks)
constexpr int kDecodeSpanMin = 256, kDecodeSpanMax = 4096;
int attn_decode_span(int batch, int n_kv_heads);
// once per decode step: the compact list of work items (request, span, tokens to attend to, 0),
// its unused tail marked with request -1 up to attn_decode_items(), and per item the physical pages
// of its span (span_len / 16 entries each)
int attn_decode_items(int batch, int max_spans, int span_len);
hipError_t launch_attn_plan(const int32_t* ctx_lens, const int32_t* block_tables, int max_pages_per_seq, int batch,
                            int max_spans, int span_len, int4* items, int32_t* n_items, int32_t* item_pages,
                            hipStream_t s);
// the attention kernel proper: finishes every request whose context fits one span, leaves fp32 partials
// (part_o, part_ml) for the others ...
hipError_t launch_attn_decode(const void* qkv, int64_t ld, int batch, int n_q_heads, const KvLayout& kv,
                              const int4* items, const int32_t* item_pages, float* part_o, float* part_ml,
                              int max_spans, int span_len, void* out, OperandLayout out_layout, hipStream_t s);
// ... which this combines (a no-op launch-wise when no request can have more than one span)
hipError_t launch_attn_decode_merge(int batch, int n_q_heads, const KvLayout& kv, const int32_t* ctx_lens,
                                    const float* part_o, const float* part_ml, int max_spans, int span_len, void* out,
                                    OperandLayout out_layout, hipStream_t s);
// diagnostic: dst[i] = E4M3 code of src[i] / scale (to_codes) or dst[i] = value of code src[i] (fp32), through the
// same device functions the KV kernels use (the decode direction through the hardware conversion)
hipError_t launch_e4m3_convert(int to_codes, const void* src, void* dst, int64_t n, float scale, hipStream_t s);
hipError_t launch_attn_prefill(const void* qkv, int64_t ld, int total_tokens, int n_seqs, int n_q_heads,
                               const KvLayout& kv, const int32_t* cu_seqlens, const int32_t* block_tables,
                               int max_pages_per_seq, void* out, OperandLayout out_layout, hipStream_t s);

}  // namespace tdp
