// C ABI of the stage library: configuration checks, memory ownership, weight repack and the
// per-layer kernel sequence of the prefill and decode phases.  See include/tdp.h for the contract.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <string>
#include <vector>

#include "../../include/tdp.h"
#include "tdp_kernels.h"

using namespace tdp;

namespace {

thread_local std::string g_err;

int fail(int code, const std::string& msg) {
  g_err = msg;
  return code;
}
int fail_hip(hipError_t e, const char* what) {
  g_err = std::string(what) + ": " + hipGetErrorString(e);
  return e == hipErrorOutOfMemory ? TDP_ENOMEM : TDP_EHIP;
}
#define HIP_TRY(expr)                                   \
  do {                                                  \
    hipError_t e__ = (expr);                            \
    if (e__ != hipSuccess) return fail_hip(e__, #expr); \
  } while (0)

int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }

enum TimeClass { T_NORM = 0, T_QKV, T_ROPE, T_ATTN, T_O, T_GU, T_DOWN, T_MERGE, T_COUNT };

}  // namespace

namespace tdp {
// the error channel for the entry points that live in other files of the library
int probe_fail(int code, const char* msg) { return fail(code, msg); }
}  // namespace tdp

struct tdp_stage {
  tdp_stage_config cfg;
  int64_t dq, Nqkv, Nqkv_pad, d_pad, Fpad, Ngu_pad;
  uint16_t *wqkv = nullptr, *wo = nullptr, *wgu = nullptr, *wd = nullptr;  // bf16 bits
  float *g_attn = nullptr, *g_mlp = nullptr;
  float* bqkv = nullptr;  // [L][Nqkv_pad]: q / k / v projection biases, zero until set
  bool has_bias = false;
  uint8_t *kpool = nullptr, *vpool = nullptr;
  int64_t pool_elems = 0;  // per layer, per pool
  int64_t pool_bytes = 0;  // pool_elems * (2: bf16 | 1: E4M3 codes)
  float k_scale = 1.f, v_scale = 1.f;
  // Everything one pass over a batch writes besides the KV pools.  A stage that runs decode batches as two
  // half-batches on two streams (decode_micro_batches = 2) holds two sets.
  struct Scratch {
    uint16_t *y = nullptr, *qkv = nullptr, *attn = nullptr, *u = nullptr;  // bf16 activations
    float* qkv32 = nullptr;  // the QKV projection as the GEMM leaves it (fp32): rotated before its one rounding
    float *h = nullptr, *xa = nullptr, *xb = nullptr;  // residual stream, fp32 between layers
    float* ws = nullptr;
    float *part_o = nullptr, *part_ml = nullptr;
    int4* attn_items = nullptr;     // decode work list, rebuilt every step
    int32_t* attn_n_items = nullptr;
    int32_t* attn_item_pages = nullptr;  // physical pages of every item's span
  };
  Scratch sc[2];
  int n_scratch = 1;
  hipStream_t aux_stream = nullptr;             // second half-batch (default priority)
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  int64_t ws_elems = 0;
  int max_chunks = 0;             // spans of kDecodeSpanMin tokens in the longest context
  float2* rope_table = nullptr;
  int32_t *check_owner = nullptr, *check_res = nullptr;  // scratch of the table checks
  int max_pos = 0;
  int maxM = 0;
  int layer_first = 0, layer_count = 0;  // count 0 = all layers
  int decode_span = 0;                   // 0 = chosen from the batch size
  bool timing = false;
  std::vector<hipEvent_t> ev_start, ev_stop;
  std::vector<int> ev_class;
  size_t ev_used = 0;
};

namespace {

int check_config(const tdp_stage_config* c) {
  if (!c) return fail(TDP_EINVAL, "config is null");
  if (c->n_layers < 1) return fail(TDP_EINVAL, "n_layers must be >= 1");
  if (c->d_model < 64 || c->d_model % 64) return fail(TDP_EINVAL, "d_model must be a positive multiple of 64");
  if (c->head_dim != 64 && c->head_dim != 128) return fail(TDP_EINVAL, "head_dim must be 64 or 128");
  if (c->n_kv_heads < 1 || c->n_q_heads < 1) return fail(TDP_EINVAL, "head counts must be >= 1");
  if (c->n_q_heads % c->n_kv_heads) return fail(TDP_EINVAL, "n_q_heads must be a multiple of n_kv_heads");
  if (c->n_q_heads / c->n_kv_heads > 16) return fail(TDP_EINVAL, "GQA group size above 16 is not supported");
  if (c->d_ff < 4 || c->d_ff % 4) return fail(TDP_EINVAL, "d_ff must be a positive multiple of 4");
  if (!(c->rms_eps >= 0.f) || !(c->rope_base > 0.f)) return fail(TDP_EINVAL, "rms_eps must be >= 0 and rope_base > 0");
  if (c->page_size != 16) return fail(TDP_EINVAL, "page_size must be 16");
  if (c->num_pages < 1) return fail(TDP_EINVAL, "num_pages must be >= 1");
  if (c->max_batch < 0 || c->max_tokens < 0 || (c->max_batch == 0 && c->max_tokens == 0))
    return fail(TDP_EINVAL, "max_batch / max_tokens must be >= 0 and not both 0");
  if (c->max_seqs < 0 || (c->max_tokens > 0 && c->max_seqs < 1))
    return fail(TDP_EINVAL, "max_seqs must be >= 1 when max_tokens > 0");
  if (c->max_pages_per_seq < 1) return fail(TDP_EINVAL, "max_pages_per_seq must be >= 1");
  if ((int64_t)c->max_pages_per_seq * 16 > (1 << 20)) return fail(TDP_EINVAL, "max_pages_per_seq too large");
  if (c->decode_micro_batches < 0 || c->decode_micro_batches > 2)
    return fail(TDP_EINVAL, "decode_micro_batches must be 0, 1 or 2");
  if (c->kv_dtype != TDP_KV_BF16 && c->kv_dtype != TDP_KV_FP8_E4M3)
    return fail(TDP_EINVAL, "kv_dtype must be TDP_KV_BF16 or TDP_KV_FP8_E4M3");
  if (c->kv_dtype == TDP_KV_FP8_E4M3) {
    // 0 means 1; otherwise a finite positive number
    if (!(c->k_scale >= 0.f) || !(c->v_scale >= 0.f) || !(c->k_scale < 1e30f) || !(c->v_scale < 1e30f))
      return fail(TDP_EINVAL, "k_scale / v_scale must be finite and >= 0 (0 = 1)");
  }
  return TDP_OK;
}

template <typename T>
hipError_t dev_alloc(T** p, int64_t elems, bool zero) {
  hipError_t e = hipMalloc((void**)p, (size_t)(elems > 0 ? elems : 1) * sizeof(T));
  if (e != hipSuccess) return e;
  if (zero) e = hipMemset(*p, 0, (size_t)(elems > 0 ? elems : 1) * sizeof(T));
  return e;
}

struct Timer {
  tdp_stage* st;
  hipStream_t s;
  bool on;
  Timer(tdp_stage* st_, hipStream_t s_, bool timed, int cls) : st(st_), s(s_), on(st_->timing && timed) {
    if (!on) return;
    if (st->ev_used == st->ev_start.size()) {
      hipEvent_t a, b;
      if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) {
        on = false;
        return;
      }
      st->ev_start.push_back(a);
      st->ev_stop.push_back(b);
      st->ev_class.push_back(cls);
    }
    st->ev_class[st->ev_used] = cls;
    (void)hipEventRecord(st->ev_start[st->ev_used], s);
  }
  ~Timer() {
    if (!on) return;
    (void)hipEventRecord(st->ev_stop[st->ev_used], s);
    st->ev_used++;
  }
};

KvLayout kv_layout(tdp_stage* st, int layer) {
  KvLayout kv;
  kv.k_pool = st->kpool + (int64_t)layer * st->pool_bytes;
  kv.v_pool = st->vpool + (int64_t)layer * st->pool_bytes;
  kv.fp8 = st->cfg.kv_dtype == TDP_KV_FP8_E4M3;
  kv.k_scale = st->k_scale;
  kv.v_scale = st->v_scale;
  kv.num_pages = st->cfg.num_pages;
  kv.n_kv_heads = st->cfg.n_kv_heads;
  kv.head_dim = st->cfg.head_dim;
  kv.page_size = 16;
  return kv;
}

// The layer sequence shared by both phases.  M tokens; decode when ctx_lens != null.
int run_layers(tdp_stage* st, tdp_stage::Scratch& sc, bool timed, const void* hidden_in, void* hidden_out, int M,
               const int32_t* ctx_lens, const int32_t* cu_seqlens, int n_seqs, const int32_t* block_tables,
               hipStream_t s) {
  const tdp_stage_config& c = st->cfg;
  const int64_t d = c.d_model;
  if (timed) st->ev_used = 0;
  // The residual stream enters and leaves the stage as bf16 (the pipeline's hand-over format) and
  // is kept in fp32 in between: two bf16 roundings per layer would otherwise pile up over a
  // 20-layer stage to more than the 2e-2 parity bound.
  const void* x = hidden_in;
  int x_f32 = 0;
  const int span_len = st->decode_span > 0 ? st->decode_span : attn_decode_span(M, c.n_kv_heads);
  if (ctx_lens)
    HIP_TRY(launch_attn_plan(ctx_lens, block_tables, c.max_pages_per_seq, M, st->max_chunks, span_len, sc.attn_items,
                             sc.attn_n_items, sc.attn_item_pages, s));
  const int l_begin = st->layer_count > 0 ? st->layer_first : 0;
  const int l_end = st->layer_count > 0 ? st->layer_first + st->layer_count : c.n_layers;
  // A projection whose K range was split leaves fp32 partials in the workspace; the kernel that
  // consumes its output sums them (RoPE for QKV, the following RMSNorm for the two residual
  // projections), which saves a reduce launch and one round trip of the result per projection.
  // (measured on the 70B-shaped stage with 1024 threads per row: +1.3 % at 16 rows, +1.7 % at 128, +1.6 % at 512)
  const bool fuse_reduce = true;
  int down_splits = 1;  // > 1: x (this layer's input) still has to be formed from h + partials
  for (int l = l_begin; l < l_end; ++l) {
    const KvLayout kv = kv_layout(st, l);
    const bool last = l == l_end - 1;
    void* x_next = last ? hidden_out : (void*)((l & 1) ? sc.xb : sc.xa);
    {  // a1: pre-attention RMSNorm
      Timer t(st, s, timed, T_NORM);
      if (down_splits > 1)
        HIP_TRY(launch_rmsnorm_sum(sc.h, 1, d, sc.ws, down_splits, st->d_pad, (float*)const_cast<void*>(x), d,
                                   st->g_attn + (int64_t)l * d, c.rms_eps, M, (int)d, sc.y, layout_paired(d), s));
      else
        HIP_TRY(launch_rmsnorm(x, x_f32, d, st->g_attn + (int64_t)l * d, c.rms_eps, M, (int)d, sc.y, layout_paired(d), s));
    }
    GemmArgs g;
    memset(&g, 0, sizeof(g));
    int qkv_splits = 1, o_splits = 1;
    g.workspace = sc.ws;
    g.workspace_elems = st->ws_elems;
    g.M = M;
    {  // a2: fused QKV projection
      Timer t(st, s, timed, T_QKV);
      g.A = sc.y; g.a_layout = layout_paired(d);
      g.W = st->wqkv + (int64_t)l * st->Nqkv_pad * d; g.Kpad = d; g.Npad = st->Nqkv_pad;
      g.N_store = (int)st->Nqkv_pad; g.out = sc.qkv32; g.ldo = st->Nqkv_pad;
      g.residual = nullptr; g.ldr = 0; g.epilogue = EPI_STORE; g.out_f32 = 1; g.residual_f32 = 0;
      g.bias = st->has_bias ? st->bqkv + (int64_t)l * st->Nqkv_pad : nullptr;
      g.splits_used = fuse_reduce ? &qkv_splits : nullptr;
      HIP_TRY(launch_gemm(g, s));
      g.splits_used = nullptr;
    }
    {  // a3: rotary embedding + KV append, from the fp32 projection (if it was split: sums the partials and
       // adds the bias, which the GEMM's epilogue has done otherwise)
      Timer t(st, s, timed, T_ROPE);
      const bool split = qkv_splits > 1;
      HIP_TRY(launch_rope_kv(sc.qkv, st->Nqkv_pad, M, c.n_q_heads, kv, st->rope_table, st->max_pos, ctx_lens,
                             cu_seqlens, n_seqs, block_tables, c.max_pages_per_seq, split ? sc.ws : sc.qkv32,
                             qkv_splits, split ? g.bias : nullptr, s));
      g.bias = nullptr;
    }
    {  // a4: attention
      Timer t(st, s, timed, T_ATTN);
      if (ctx_lens)
        HIP_TRY(launch_attn_decode(sc.qkv, st->Nqkv_pad, M, c.n_q_heads, kv, sc.attn_items, sc.attn_item_pages,
                                   sc.part_o, sc.part_ml, st->max_chunks, span_len, sc.attn, layout_paired(st->dq), s));
      else
        HIP_TRY(launch_attn_prefill(sc.qkv, st->Nqkv_pad, M, n_seqs, c.n_q_heads, kv, cu_seqlens, block_tables,
                                    c.max_pages_per_seq, sc.attn, layout_paired(st->dq), s));
    }
    if (ctx_lens) {  // a4, second kernel: requests longer than one span are combined from their partials
      Timer t(st, s, timed, T_MERGE);
      HIP_TRY(launch_attn_decode_merge(M, c.n_q_heads, kv, ctx_lens, sc.part_o, sc.part_ml, st->max_chunks, span_len,
                                       sc.attn, layout_paired(st->dq), s));
    }
    {  // a5: output projection + residual -> h (fp32)
      Timer t(st, s, timed, T_O);
      g.A = sc.attn; g.a_layout = layout_paired(st->dq);
      g.W = st->wo + (int64_t)l * st->d_pad * st->dq; g.Kpad = st->dq; g.Npad = st->d_pad;
      g.N_store = (int)d; g.out = sc.h; g.ldo = d; g.out_f32 = 1;
      g.residual = x; g.ldr = d; g.residual_f32 = x_f32; g.epilogue = EPI_RESIDUAL;
      g.splits_used = fuse_reduce ? &o_splits : nullptr;
      HIP_TRY(launch_gemm(g, s));
      g.splits_used = nullptr;
    }
    {  // a6: pre-MLP RMSNorm (forms h = x + partials first if the projection was split)
      Timer t(st, s, timed, T_NORM);
      if (o_splits > 1)
        HIP_TRY(launch_rmsnorm_sum(x, x_f32, d, sc.ws, o_splits, st->d_pad, sc.h, d, st->g_mlp + (int64_t)l * d,
                                   c.rms_eps, M, (int)d, sc.y, layout_paired(d), s));
      else
        HIP_TRY(launch_rmsnorm(sc.h, 1, d, st->g_mlp + (int64_t)l * d, c.rms_eps, M, (int)d, sc.y, layout_paired(d), s));
    }
    {  // a7: gate/up projection + SwiGLU
      Timer t(st, s, timed, T_GU);
      g.A = sc.y; g.a_layout = layout_paired(d);
      g.W = st->wgu + (int64_t)l * st->Ngu_pad * d; g.Kpad = d; g.Npad = st->Ngu_pad;
      g.N_store = (int)st->Fpad; g.out = sc.u; g.ldo = st->Fpad; g.u_layout = layout_paired(st->Fpad); g.out_f32 = 0;
      g.residual = nullptr; g.ldr = 0; g.residual_f32 = 0; g.epilogue = EPI_SWIGLU;
      HIP_TRY(launch_gemm(g, s));
    }
    {  // a8: down projection + residual -> next layer's stream (fp32), or the stage output (bf16)
      Timer t(st, s, timed, T_DOWN);
      g.A = sc.u; g.a_layout = layout_paired(st->Fpad);
      g.W = st->wd + (int64_t)l * st->d_pad * st->Fpad; g.Kpad = st->Fpad; g.Npad = st->d_pad;
      g.N_store = (int)d; g.out = x_next; g.ldo = d; g.out_f32 = last ? 0 : 1;
      g.residual = sc.h; g.ldr = d; g.residual_f32 = 1; g.epilogue = EPI_RESIDUAL;
      down_splits = 1;
      g.splits_used = last || !fuse_reduce ? nullptr : &down_splits;  // the stage output has no norm behind it
      HIP_TRY(launch_gemm(g, s));
      g.splits_used = nullptr;
    }
    x = x_next;
    x_f32 = 1;
  }
  return TDP_OK;
}

}  // namespace

extern "C" {

int tdp_abi_version(void) { return 5; }

const char* tdp_last_error(void) { return g_err.c_str(); }

int tdp_stage_create(const tdp_stage_config* cfg, tdp_stage** out) {
  if (!out) return fail(TDP_EINVAL, "out is null");
  int rc = check_config(cfg);
  if (rc != TDP_OK) return rc;
  tdp_stage* st = new (std::nothrow) tdp_stage();
  if (!st) return fail(TDP_ENOMEM, "host allocation failed");
  st->cfg = *cfg;
  const tdp_stage_config& c = st->cfg;
  const int64_t d = c.d_model, dh = c.head_dim, L = c.n_layers;
  st->dq = (int64_t)c.n_q_heads * dh;
  st->Nqkv = st->dq + 2 * (int64_t)c.n_kv_heads * dh;
  st->Nqkv_pad = round_up(st->Nqkv, 256);
  st->d_pad = round_up(d, 256);
  st->Fpad = round_up(c.d_ff, 128);
  st->Ngu_pad = 2 * st->Fpad;
  st->maxM = c.max_batch > c.max_tokens ? c.max_batch : c.max_tokens;
  st->pool_elems = (int64_t)c.num_pages * c.n_kv_heads * 16 * dh;
  st->pool_bytes = st->pool_elems * (c.kv_dtype == TDP_KV_FP8_E4M3 ? 1 : 2);
  if (c.kv_dtype == TDP_KV_FP8_E4M3) {
    st->k_scale = c.k_scale > 0.f ? c.k_scale : 1.f;
    st->v_scale = c.v_scale > 0.f ? c.v_scale : 1.f;
  }
  st->max_pos = c.max_pages_per_seq * 16;
  st->max_chunks = (st->max_pos + kDecodeSpanMin - 1) / kDecodeSpanMin;

  hipError_t e = gemm_setup();
  auto A = [&](auto** p, int64_t n, bool zero) {
    if (e == hipSuccess) e = dev_alloc(p, n, zero);
  };
  A(&st->wqkv, L * st->Nqkv_pad * d, true);
  A(&st->wo, L * st->d_pad * st->dq, true);
  A(&st->wgu, L * st->Ngu_pad * d, true);
  A(&st->wd, L * st->d_pad * st->Fpad, true);
  A(&st->g_attn, L * d, true);
  A(&st->g_mlp, L * d, true);
  A(&st->bqkv, L * st->Nqkv_pad, true);
  A(&st->kpool, L * st->pool_bytes, true);
  A(&st->vpool, L * st->pool_bytes, true);
  st->n_scratch = c.decode_micro_batches == 2 ? 2 : 1;
  // the second set only ever holds half a decode batch
  for (int i = 0; i < st->n_scratch; ++i) {
    tdp_stage::Scratch& sc = st->sc[i];
    const int64_t rows = i == 0 ? st->maxM : (c.max_batch + 1) / 2;
    const int64_t M = (rows + 1) & ~1;  // row pairs: pair-interleaved activation buffers
    const int64_t mb = i == 0 ? c.max_batch : (c.max_batch + 1) / 2;
    A(&sc.y, M * d, true);
    A(&sc.qkv, M * st->Nqkv_pad, true);
    A(&sc.qkv32, M * st->Nqkv_pad, true);
    A(&sc.attn, M * st->dq, true);
    A(&sc.h, M * d, true);
    A(&sc.u, M * st->Fpad, true);
    A(&sc.xa, M * d, true);
    A(&sc.xb, M * d, true);
    {
      int64_t maxN = st->Ngu_pad > st->Nqkv_pad ? st->Ngu_pad : st->Nqkv_pad;
      if (st->d_pad > maxN) maxN = st->d_pad;
      const int64_t mdec = st->maxM + 1 < 512 ? ((st->maxM + 1) & ~1) : 512;
      st->ws_elems = 8 * mdec * maxN;
      if (st->ws_elems > (64ll << 20)) st->ws_elems = 64ll << 20;
      A(&sc.ws, st->ws_elems, false);
    }
    A(&sc.part_o, mb * c.n_q_heads * st->max_chunks * dh, false);
    A(&sc.part_ml, mb * c.n_q_heads * st->max_chunks * 2, false);
    A(&sc.attn_items, mb * st->max_chunks, false);
    // spans longer than the minimum round the span count up: up to (1024 / 256 - 1) extra minimum spans' worth
    A(&sc.attn_item_pages, mb * (st->max_chunks + kDecodeSpanMax / kDecodeSpanMin) * (kDecodeSpanMin / 16), false);
    A(&sc.attn_n_items, 1, true);
  }
  if (e == hipSuccess && st->n_scratch == 2) {
    e = hipStreamCreateWithFlags(&st->aux_stream, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&st->ev_fork, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&st->ev_join, hipEventDisableTiming);
  }
  A(&st->rope_table, (int64_t)st->max_pos * (dh / 2), false);
  A(&st->check_owner, c.num_pages, false);
  A(&st->check_res, 2, true);
  if (e == hipSuccess) {
    // (cos, sin)(pos * base^(-2i/dh)) in double precision, stored as fp32
    std::vector<float2> tab((size_t)st->max_pos * (dh / 2));
    for (int64_t p = 0; p < st->max_pos; ++p)
      for (int64_t i = 0; i < dh / 2; ++i) {
        const double theta = pow((double)c.rope_base, -2.0 * (double)i / (double)dh);
        const double ang = (double)p * theta;
        tab[p * (dh / 2) + i] = make_float2((float)cos(ang), (float)sin(ang));
      }
    e = hipMemcpy(st->rope_table, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice);
  }
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    int code = fail_hip(e, "tdp_stage_create");
    tdp_stage_destroy(st);
    return code;
  }
  *out = st;
  return TDP_OK;
}

void tdp_stage_destroy(tdp_stage* st) {
  if (!st) return;
  (void)hipDeviceSynchronize();
  void* ptrs[] = {st->wqkv, st->wo, st->wgu, st->wd, st->g_attn, st->g_mlp, st->bqkv, st->kpool, st->vpool,
                  st->rope_table, st->check_owner, st->check_res};
  for (void* p : ptrs)
    if (p) (void)hipFree(p);
  for (tdp_stage::Scratch& sc : st->sc) {
    void* sp[] = {sc.y, sc.qkv, sc.qkv32, sc.attn, sc.h, sc.u, sc.xa, sc.xb, sc.ws, sc.part_o, sc.part_ml, sc.attn_items,
                  sc.attn_n_items, sc.attn_item_pages};
    for (void* p : sp)
      if (p) (void)hipFree(p);
  }
  if (st->ev_fork) (void)hipEventDestroy(st->ev_fork);
  if (st->ev_join) (void)hipEventDestroy(st->ev_join);
  if (st->aux_stream) (void)hipStreamDestroy(st->aux_stream);
  for (hipEvent_t ev : st->ev_start) (void)hipEventDestroy(ev);
  for (hipEvent_t ev : st->ev_stop) (void)hipEventDestroy(ev);
  delete st;
}

int tdp_stage_set_weight(tdp_stage* st, int32_t layer, int32_t which, const void* src, int32_t dtype,
                         int32_t mem, int64_t rows, int64_t cols) {
  if (!st || !src) return fail(TDP_EINVAL, "null stage or source");
  const tdp_stage_config& c = st->cfg;
  if (layer < 0 || layer >= c.n_layers) return fail(TDP_EINVAL, "layer out of range");
  if (dtype != TDP_F32 && dtype != TDP_BF16) return fail(TDP_EINVAL, "dtype must be TDP_F32 or TDP_BF16");
  if (mem != TDP_HOST && mem != TDP_DEVICE) return fail(TDP_EINVAL, "mem must be TDP_HOST or TDP_DEVICE");
  const int64_t d = c.d_model, dkv = (int64_t)c.n_kv_heads * c.head_dim, F = c.d_ff;
  int64_t er = 0, ec = 0;
  switch (which) {
    case TDP_WQ: er = d; ec = st->dq; break;
    case TDP_WK: case TDP_WV: er = d; ec = dkv; break;
    case TDP_WO: er = st->dq; ec = d; break;
    case TDP_WG: case TDP_WU: er = d; ec = F; break;
    case TDP_WD: er = F; ec = d; break;
    case TDP_G_ATTN: case TDP_G_MLP: er = d; ec = 1; break;
    case TDP_BQ: er = st->dq; ec = 1; break;
    case TDP_BK: case TDP_BV: er = dkv; ec = 1; break;
    default: return fail(TDP_EINVAL, "unknown weight id");
  }
  if (rows != er || cols != ec) {
    char buf[160];
    snprintf(buf, sizeof buf, "weight %d expects [%lld, %lld], got [%lld, %lld]", which, (long long)er,
             (long long)ec, (long long)rows, (long long)cols);
    return fail(TDP_EINVAL, buf);
  }
  const size_t esz = dtype == TDP_F32 ? 4 : 2;
  const void* dsrc = src;
  void* tmp = nullptr;
  if (mem == TDP_HOST) {
    HIP_TRY(hipMalloc(&tmp, (size_t)(rows * cols) * esz));
    hipError_t e = hipMemcpy(tmp, src, (size_t)(rows * cols) * esz, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
      (void)hipFree(tmp);
      return fail_hip(e, "hipMemcpy(weight)");
    }
    dsrc = tmp;
  }
  const int f32 = dtype == TDP_F32;
  hipError_t e = hipSuccess;
  switch (which) {
    case TDP_WQ:
      e = launch_repack(dsrc, f32, rows, cols, st->wqkv + (int64_t)layer * st->Nqkv_pad * d, d, 0, 0, 0); break;
    case TDP_WK:
      e = launch_repack(dsrc, f32, rows, cols, st->wqkv + (int64_t)layer * st->Nqkv_pad * d, d, st->dq, 0, 0); break;
    case TDP_WV:
      e = launch_repack(dsrc, f32, rows, cols, st->wqkv + (int64_t)layer * st->Nqkv_pad * d, d, st->dq + dkv, 0, 0); break;
    case TDP_WO:
      e = launch_repack(dsrc, f32, rows, cols, st->wo + (int64_t)layer * st->d_pad * st->dq, st->dq, 0, 0, 0); break;
    case TDP_WG:
      e = launch_repack(dsrc, f32, rows, cols, st->wgu + (int64_t)layer * st->Ngu_pad * d, d, 0, 1, 0); break;
    case TDP_WU:
      e = launch_repack(dsrc, f32, rows, cols, st->wgu + (int64_t)layer * st->Ngu_pad * d, d, 0, 2, 0); break;
    case TDP_WD:
      e = launch_repack(dsrc, f32, rows, cols, st->wd + (int64_t)layer * st->d_pad * st->Fpad, st->Fpad, 0, 0, 0); break;
    case TDP_G_ATTN:
      e = launch_convert_vec(dsrc, f32, d, st->g_attn + (int64_t)layer * d, 0); break;
    case TDP_BQ:
      e = launch_convert_vec(dsrc, f32, st->dq, st->bqkv + (int64_t)layer * st->Nqkv_pad, 0);
      st->has_bias = true; break;
    case TDP_BK:
      e = launch_convert_vec(dsrc, f32, dkv, st->bqkv + (int64_t)layer * st->Nqkv_pad + st->dq, 0);
      st->has_bias = true; break;
    case TDP_BV:
      e = launch_convert_vec(dsrc, f32, dkv, st->bqkv + (int64_t)layer * st->Nqkv_pad + st->dq + dkv, 0);
      st->has_bias = true; break;
    default:
      e = launch_convert_vec(dsrc, f32, d, st->g_mlp + (int64_t)layer * d, 0); break;
  }
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (tmp) (void)hipFree(tmp);
  if (e != hipSuccess) return fail_hip(e, "weight repack");
  return TDP_OK;
}

int tdp_stage_kv_pool(tdp_stage* st, int32_t layer, void** k_dev, void** v_dev, int64_t* bytes) {
  if (!st) return fail(TDP_EINVAL, "null stage");
  if (layer < 0 || layer >= st->cfg.n_layers) return fail(TDP_EINVAL, "layer out of range");
  if (k_dev) *k_dev = st->kpool + (int64_t)layer * st->pool_bytes;
  if (v_dev) *v_dev = st->vpool + (int64_t)layer * st->pool_bytes;
  if (bytes) *bytes = st->pool_bytes;
  return TDP_OK;
}

static int kv_copy_common(int to_pages, tdp_stage* st, int32_t layer, void* k_packed, void* v_packed,
                          const int32_t* cu_seqlens, const int32_t* block_tables, int32_t n_seqs,
                          int32_t total_tokens, void* stream) {
  if (!st) return fail(TDP_EINVAL, "null stage");
  if (layer < 0 || layer >= st->cfg.n_layers) return fail(TDP_EINVAL, "layer out of range");
  if (n_seqs < 0 || total_tokens < 0) return fail(TDP_EINVAL, "negative size");
  if (n_seqs == 0 || total_tokens == 0) return TDP_OK;
  if (!k_packed || !v_packed || !cu_seqlens || !block_tables) return fail(TDP_EINVAL, "null pointer");
  HIP_TRY(launch_kv_copy(to_pages, k_packed, v_packed, kv_layout(st, layer), cu_seqlens, n_seqs, total_tokens,
                         block_tables, st->cfg.max_pages_per_seq, (hipStream_t)stream));
  return TDP_OK;
}

int tdp_stage_kv_import(tdp_stage* st, int32_t layer, const void* k_packed, const void* v_packed,
                        const int32_t* cu_seqlens, const int32_t* block_tables, int32_t n_seqs,
                        int32_t total_tokens, void* stream) {
  return kv_copy_common(1, st, layer, (void*)k_packed, (void*)v_packed, cu_seqlens, block_tables, n_seqs,
                        total_tokens, stream);
}

int tdp_stage_kv_export(tdp_stage* st, int32_t layer, void* k_packed, void* v_packed,
                        const int32_t* cu_seqlens, const int32_t* block_tables, int32_t n_seqs,
                        int32_t total_tokens, void* stream) {
  return kv_copy_common(0, st, layer, k_packed, v_packed, cu_seqlens, block_tables, n_seqs, total_tokens,
                        stream);
}

int tdp_stage_prefill(tdp_stage* st, const void* hidden_in, const int32_t* cu_seqlens,
                      const int32_t* block_tables, int32_t n_seqs, int32_t total_tokens, void* hidden_out,
                      void* stream) {
  if (!st) return fail(TDP_EINVAL, "null stage");
  if (n_seqs < 0 || total_tokens < 0) return fail(TDP_EINVAL, "negative size");
  if (n_seqs > st->cfg.max_seqs) return fail(TDP_EINVAL, "n_seqs exceeds max_seqs");
  if (total_tokens > st->cfg.max_tokens) return fail(TDP_EINVAL, "total_tokens exceeds max_tokens");
  if (n_seqs == 0 || total_tokens == 0) return TDP_OK;
  if (!hidden_in || !hidden_out || !cu_seqlens || !block_tables) return fail(TDP_EINVAL, "null pointer");
  return run_layers(st, st->sc[0], true, hidden_in, hidden_out, total_tokens, nullptr, cu_seqlens, n_seqs, block_tables,
                    (hipStream_t)stream);
}

int tdp_stage_decode(tdp_stage* st, const void* hidden_in, const int32_t* ctx_lens, const int32_t* block_tables,
                     int32_t batch, void* hidden_out, void* stream) {
  if (!st) return fail(TDP_EINVAL, "null stage");
  if (batch < 0) return fail(TDP_EINVAL, "negative batch");
  if (batch > st->cfg.max_batch) return fail(TDP_EINVAL, "batch exceeds max_batch");
  if (batch == 0) return TDP_OK;
  if (!hidden_in || !hidden_out || !ctx_lens || !block_tables) return fail(TDP_EINVAL, "null pointer");
  hipStream_t s = (hipStream_t)stream;
  if (st->n_scratch < 2 || batch < 2)
    return run_layers(st, st->sc[0], true, hidden_in, hidden_out, batch, ctx_lens, nullptr, batch, block_tables, s);
  // Two half-batches, one on the caller's stream and one on the stage's second stream, so that one half's
  // attention (bound by reading the cache, Sec. 2.1) can run beside the other half's projections.  The
  // second stream starts after everything already queued on the caller's stream and is joined at the end.
  const int half = (batch + 1) / 2;
  const int64_t d = st->cfg.d_model;
  st->ev_used = 0;  // per-class timing is not recorded for the two-stream form
  HIP_TRY(hipEventRecord(st->ev_fork, s));
  HIP_TRY(hipStreamWaitEvent(st->aux_stream, st->ev_fork, 0));
  int rc = run_layers(st, st->sc[0], false, hidden_in, hidden_out, half, ctx_lens, nullptr, half, block_tables, s);
  if (rc != TDP_OK) return rc;
  rc = run_layers(st, st->sc[1], false, (const uint16_t*)hidden_in + (int64_t)half * d,
                  (uint16_t*)hidden_out + (int64_t)half * d, batch - half, ctx_lens + half, nullptr, batch - half,
                  block_tables + (int64_t)half * st->cfg.max_pages_per_seq, st->aux_stream);
  if (rc != TDP_OK) return rc;
  HIP_TRY(hipEventRecord(st->ev_join, st->aux_stream));
  HIP_TRY(hipStreamWaitEvent(s, st->ev_join, 0));
  return TDP_OK;
}

static int check_tables(tdp_stage* st, int decode, const int32_t* lens, const int32_t* block_tables, int n_rows,
                        int total_tokens, hipStream_t s) {
  HIP_TRY(launch_table_check(decode, lens, block_tables, n_rows, st->cfg.max_pages_per_seq, st->cfg.num_pages,
                             total_tokens, st->check_owner, st->check_res, s));
  int32_t res[2] = {0, 0};
  HIP_TRY(hipMemcpyAsync(res, st->check_res, sizeof res, hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  if (res[0] == 0) return TDP_OK;
  const int row = res[1] / 8, kind = res[1] % 8;
  static const char* const what[] = {
      "", "length outside what a block-table row can hold", "page id outside [0, num_pages)",
      "a page this call writes appears more than once in the batch", "cu_seqlens does not run from 0 to total_tokens"};
  char buf[200];
  snprintf(buf, sizeof buf, "%d table violation(s); first: row %d, %s", (int)res[0], row,
           kind >= 1 && kind <= 4 ? what[kind] : "unknown");
  return fail(TDP_EINVAL, buf);
}

int tdp_stage_check_decode(tdp_stage* st, const int32_t* ctx_lens, const int32_t* block_tables, int32_t batch,
                           void* stream) {
  if (!st) return fail(TDP_EINVAL, "null stage");
  if (batch < 0) return fail(TDP_EINVAL, "negative batch");
  if (batch > st->cfg.max_batch) return fail(TDP_EINVAL, "batch exceeds max_batch");
  if (batch == 0) return TDP_OK;
  if (!ctx_lens || !block_tables) return fail(TDP_EINVAL, "null pointer");
  return check_tables(st, 1, ctx_lens, block_tables, batch, 0, (hipStream_t)stream);
}

int tdp_stage_check_prefill(tdp_stage* st, const int32_t* cu_seqlens, const int32_t* block_tables, int32_t n_seqs,
                            int32_t total_tokens, void* stream) {
  if (!st) return fail(TDP_EINVAL, "null stage");
  if (n_seqs < 0 || total_tokens < 0) return fail(TDP_EINVAL, "negative size");
  if (n_seqs > st->cfg.max_seqs) return fail(TDP_EINVAL, "n_seqs exceeds max_seqs");
  if (total_tokens > st->cfg.max_tokens) return fail(TDP_EINVAL, "total_tokens exceeds max_tokens");
  if (n_seqs == 0 || total_tokens == 0) return TDP_OK;
  if (!cu_seqlens || !block_tables) return fail(TDP_EINVAL, "null pointer");
  return check_tables(st, 0, cu_seqlens, block_tables, n_seqs, total_tokens, (hipStream_t)stream);
}

int tdp_gemm_bf16(const void* A, const void* W, const void* residual, void* out, int32_t M, int32_t N, int32_t K,
                  int32_t epilogue, int32_t tile, int32_t splits, void* stream) {
  if (M < 0 || N <= 0 || K <= 0) return fail(TDP_EINVAL, "bad GEMM shape");
  if (K % 64 || N % 4) return fail(TDP_EINVAL, "K must be a multiple of 64 and N of 4");
  if (epilogue < 0 || epilogue > 2) return fail(TDP_EINVAL, "epilogue must be 0, 1 or 2");
  if (epilogue == 2 && N % 8) return fail(TDP_EINVAL, "the gated epilogue needs N = 2 F with F a multiple of 4");
  if (tile < 0 || tile > kGemmTileMax || splits < 0) return fail(TDP_EINVAL, "bad tile / splits");
  if (M == 0) return TDP_OK;
  if (!A || !W || !out || (epilogue == 1 && !residual)) return fail(TDP_EINVAL, "null pointer");
  hipStream_t s = (hipStream_t)stream;
  HIP_TRY(gemm_setup());
  // gated: the weights are stored as the stage stores gate/up (blocks of 32 gate rows, 32 up rows; F rounded up
  // to 128), the result has F = N / 2 columns
  const int64_t F = N / 2;
  const int64_t Npad = epilogue == 2 ? 2 * round_up(F, 128) : round_up(N, 256);
  uint16_t* wt = nullptr;
  float* ws = nullptr;
  const int64_t ws_elems = (int64_t)(splits > 0 ? splits : 16) * M * Npad;
  HIP_TRY(hipMalloc((void**)&wt, (size_t)(Npad * K) * 2));
  hipError_t e = hipMalloc((void**)&ws, (size_t)ws_elems * 4);
  if (e == hipSuccess) e = hipMemsetAsync(wt, 0, (size_t)(Npad * K) * 2, s);
  if (e == hipSuccess) {
    if (epilogue == 2) {
      // columns [0, F) of W are the gate matrix, [F, 2 F) the up matrix: each is a [K, F] matrix with leading
      // dimension N, which the repack reads through its source stride
      e = launch_repack_ld(W, 0, K, F, N, wt, K, 0, 1, s);
      if (e == hipSuccess) e = launch_repack_ld((const uint16_t*)W + F, 0, K, F, N, wt, K, 0, 2, s);
    } else {
      e = launch_repack(W, 0, K, N, wt, K, 0, 0, s);
    }
  }
  if (e == hipSuccess) {
    GemmArgs g;
    memset(&g, 0, sizeof(g));
    g.A = A; g.a_layout = layout_row_major(K); g.W = wt; g.Kpad = K; g.Npad = Npad; g.M = M;
    g.N_store = epilogue == 2 ? (int)F : N;
    g.out = out; g.ldo = g.N_store; g.u_layout = layout_row_major(F); g.residual = residual; g.ldr = N;
    g.epilogue = epilogue == 2 ? EPI_SWIGLU : epilogue ? EPI_RESIDUAL : EPI_STORE;
    g.workspace = ws; g.workspace_elems = ws_elems; g.force_tile = tile; g.force_splits = splits;
    e = launch_gemm(g, s);
  }
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (wt) (void)hipFree(wt);
  if (ws) (void)hipFree(ws);
  if (e != hipSuccess) return fail_hip(e, "tdp_gemm_bf16");
  return TDP_OK;
}

int tdp_e4m3_from_f32(const float* src, uint8_t* codes, int64_t n, float scale, void* stream) {
  if (n < 0) return fail(TDP_EINVAL, "negative size");
  if (n == 0) return TDP_OK;
  if (!src || !codes) return fail(TDP_EINVAL, "null pointer");
  if (!(scale > 0.f) || !(scale < 1e30f)) return fail(TDP_EINVAL, "scale must be finite and > 0");
  HIP_TRY(launch_e4m3_convert(1, src, codes, n, scale, (hipStream_t)stream));
  return TDP_OK;
}

int tdp_e4m3_to_f32(const uint8_t* codes, float* dst, int64_t n, void* stream) {
  if (n < 0 || n % 4) return fail(TDP_EINVAL, "n must be a non-negative multiple of 4");
  if (n == 0) return TDP_OK;
  if (!codes || !dst) return fail(TDP_EINVAL, "null pointer");
  if (((uintptr_t)codes & 3) || ((uintptr_t)dst & 15)) return fail(TDP_EINVAL, "codes must be 4-byte and dst 16-byte aligned");
  HIP_TRY(launch_e4m3_convert(0, codes, dst, n, 1.f, (hipStream_t)stream));
  return TDP_OK;
}

int tdp_stage_set_layer_range(tdp_stage* st, int32_t first, int32_t count) {
  if (!st) return fail(TDP_EINVAL, "null stage");
  if (count == 0) {
    st->layer_first = st->layer_count = 0;
    return TDP_OK;
  }
  if (first < 0 || count < 0 || first + count > st->cfg.n_layers)
    return fail(TDP_EINVAL, "layer range outside the stage");
  st->layer_first = first;
  st->layer_count = count;
  return TDP_OK;
}

int tdp_stage_set_decode_span(tdp_stage* st, int32_t span_tokens) {
  if (!st) return fail(TDP_EINVAL, "null stage");
  if (span_tokens != 0 && span_tokens != 256 && span_tokens != 512 && span_tokens != 1024 && span_tokens != 2048 &&
      span_tokens != 4096)
    return fail(TDP_EINVAL, "span must be 0 (automatic), 256, 512, 1024, 2048 or 4096 tokens");
  st->decode_span = span_tokens;
  return TDP_OK;
}

int tdp_stage_timing_enable(tdp_stage* st, int32_t on) {
  if (!st) return fail(TDP_EINVAL, "null stage");
  st->timing = on != 0;
  st->ev_used = 0;
  return TDP_OK;
}

int tdp_stage_timing_read(tdp_stage* st, float* ms) {
  if (!st || !ms) return fail(TDP_EINVAL, "null pointer");
  for (int i = 0; i < T_COUNT; ++i) ms[i] = 0.f;
  for (size_t i = 0; i < st->ev_used; ++i) {
    HIP_TRY(hipEventSynchronize(st->ev_stop[i]));
    float t = 0.f;
    HIP_TRY(hipEventElapsedTime(&t, st->ev_start[i], st->ev_stop[i]));
    ms[st->ev_class[i]] += t;
  }
  return TDP_OK;
}

// ---- the two ends of the pipeline ---------------------------------------------------------------

struct tdp_ends {
  tdp_ends_config cfg;
  int64_t v_pad = 0;
  uint16_t* table = nullptr;   // bf16 [vocab][d]
  float* gain = nullptr;       // [d]
  uint16_t* w_head = nullptr;  // bf16, pair-interleaved [v_pad][d]
  uint16_t* rows = nullptr;    // bf16 [max_tokens][d]: gathered input rows
  uint16_t* y = nullptr;       // bf16, pair-interleaved [max_tokens ^ 2][d]: normalised rows
  float* logits = nullptr;     // [max_tokens][vocab]
  float* ws = nullptr;
  int64_t ws_elems = 0;
};

int tdp_ends_create(const tdp_ends_config* cfg, tdp_ends** out) {
  if (!cfg || !out) return fail(TDP_EINVAL, "null pointer");
  if (cfg->vocab_size < 4 || cfg->vocab_size % 4) return fail(TDP_EINVAL, "vocab_size must be a positive multiple of 4");
  if (cfg->d_model < 64 || cfg->d_model % 64) return fail(TDP_EINVAL, "d_model must be a positive multiple of 64");
  if (!(cfg->rms_eps >= 0.f)) return fail(TDP_EINVAL, "rms_eps must be >= 0");
  if (cfg->max_tokens < 1) return fail(TDP_EINVAL, "max_tokens must be >= 1");
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || n_dev < 1) return fail(TDP_EHIP, "no HIP device");
  tdp_ends* e = new (std::nothrow) tdp_ends();
  if (!e) return fail(TDP_ENOMEM, "host allocation failed");
  e->cfg = *cfg;
  const int64_t d = cfg->d_model, V = cfg->vocab_size;
  e->v_pad = round_up(V, 256);
  const int64_t M = ((int64_t)cfg->max_tokens + 1) & ~1ll;
  hipError_t err = gemm_setup();
  auto A = [&](auto** p, int64_t n, bool zero) {
    if (err == hipSuccess) err = dev_alloc(p, n, zero);
  };
  A(&e->table, V * d, true);
  A(&e->gain, d, true);
  A(&e->w_head, e->v_pad * d, true);
  A(&e->rows, M * d, true);
  A(&e->y, M * d, true);
  A(&e->logits, (int64_t)cfg->max_tokens * V, false);
  e->ws_elems = 2 * (M < 512 ? M : 512) * e->v_pad;
  A(&e->ws, e->ws_elems, false);
  if (err == hipSuccess) err = hipDeviceSynchronize();
  if (err != hipSuccess) {
    const int code = fail_hip(err, "tdp_ends_create");
    tdp_ends_destroy(e);
    return code;
  }
  *out = e;
  return TDP_OK;
}

void tdp_ends_destroy(tdp_ends* e) {
  if (!e) return;
  (void)hipDeviceSynchronize();
  void* ptrs[] = {e->table, e->gain, e->w_head, e->rows, e->y, e->logits, e->ws};
  for (void* p : ptrs)
    if (p) (void)hipFree(p);
  delete e;
}

int tdp_ends_set_weight(tdp_ends* e, int32_t which, const void* src, int32_t dtype, int32_t mem, int64_t rows,
                        int64_t cols) {
  if (!e || !src) return fail(TDP_EINVAL, "null ends object or source");
  if (dtype != TDP_F32 && dtype != TDP_BF16) return fail(TDP_EINVAL, "dtype must be TDP_F32 or TDP_BF16");
  if (mem != TDP_HOST && mem != TDP_DEVICE) return fail(TDP_EINVAL, "mem must be TDP_HOST or TDP_DEVICE");
  const int64_t d = e->cfg.d_model, V = e->cfg.vocab_size;
  int64_t er, ec;
  switch (which) {
    case TDP_E_EMBEDDING: er = V; ec = d; break;
    case TDP_E_FINAL_NORM: er = d; ec = 1; break;
    case TDP_E_LM_HEAD: er = d; ec = V; break;
    default: return fail(TDP_EINVAL, "unknown weight id");
  }
  if (rows != er || cols != ec) return fail(TDP_EINVAL, "weight shape does not match the configuration");
  const size_t esz = dtype == TDP_F32 ? 4 : 2;
  const void* dsrc = src;
  void* tmp = nullptr;
  if (mem == TDP_HOST) {
    HIP_TRY(hipMalloc(&tmp, (size_t)(rows * cols) * esz));
    hipError_t err = hipMemcpy(tmp, src, (size_t)(rows * cols) * esz, hipMemcpyHostToDevice);
    if (err != hipSuccess) {
      (void)hipFree(tmp);
      return fail_hip(err, "hipMemcpy(weight)");
    }
    dsrc = tmp;
  }
  const int f32 = dtype == TDP_F32;
  hipError_t err;
  if (which == TDP_E_EMBEDDING) err = launch_to_bf16(dsrc, f32, V * d, e->table, 0);
  else if (which == TDP_E_FINAL_NORM) err = launch_convert_vec(dsrc, f32, d, e->gain, 0);
  else err = launch_repack(dsrc, f32, d, V, e->w_head, d, 0, 0, 0);
  if (err == hipSuccess) err = hipDeviceSynchronize();
  if (tmp) (void)hipFree(tmp);
  if (err != hipSuccess) return fail_hip(err, "weight conversion");
  return TDP_OK;
}

int tdp_embed_tokens(tdp_ends* e, const int32_t* token_ids, int32_t M, void* hidden_out, void* stream) {
  if (!e) return fail(TDP_EINVAL, "null ends object");
  if (M < 0) return fail(TDP_EINVAL, "negative size");
  if (M == 0) return TDP_OK;
  if (!token_ids || !hidden_out) return fail(TDP_EINVAL, "null pointer");
  HIP_TRY(launch_gather_rows(e->table, e->cfg.d_model, e->cfg.vocab_size, token_ids, M, e->cfg.d_model, hidden_out,
                             e->cfg.d_model, (hipStream_t)stream));
  return TDP_OK;
}

int tdp_lm_head(tdp_ends* e, const void* hidden_in, int32_t n_rows_in, const int32_t* row_index, int32_t M,
                float* logits_out, int32_t* next_token, void* stream) {
  if (!e) return fail(TDP_EINVAL, "null ends object");
  if (M < 0 || n_rows_in < 0) return fail(TDP_EINVAL, "negative size");
  if (M > e->cfg.max_tokens) return fail(TDP_EINVAL, "M exceeds max_tokens");
  if (M == 0) return TDP_OK;
  if (!hidden_in || n_rows_in < 1) return fail(TDP_EINVAL, "no input rows");
  if (!row_index && M > n_rows_in) return fail(TDP_EINVAL, "M exceeds the input rows");
  hipStream_t s = (hipStream_t)stream;
  const int d = e->cfg.d_model, V = e->cfg.vocab_size;
  const void* x = hidden_in;
  if (row_index) {
    HIP_TRY(launch_gather_rows(hidden_in, d, n_rows_in, row_index, M, d, e->rows, d, s));
    x = e->rows;
  }
  HIP_TRY(launch_rmsnorm(x, 0, d, e->gain, e->cfg.rms_eps, M, d, e->y, layout_paired(d), s));
  float* logits = logits_out ? logits_out : e->logits;
  GemmArgs g;
  memset(&g, 0, sizeof(g));
  g.A = e->y; g.a_layout = layout_paired(d); g.W = e->w_head; g.Kpad = d; g.Npad = e->v_pad; g.M = M; g.N_store = V;
  g.out = logits; g.ldo = V; g.epilogue = EPI_STORE; g.out_f32 = 1;
  g.workspace = e->ws; g.workspace_elems = e->ws_elems;
  HIP_TRY(launch_gemm(g, s));
  if (next_token) HIP_TRY(launch_argmax_rows(logits, V, M, V, next_token, s));
  return TDP_OK;
}

int tdp_argmax_rows(const float* logits, int32_t M, int32_t n, int64_t ld, int32_t* out, void* stream) {
  if (M < 0 || n < 1 || ld < n) return fail(TDP_EINVAL, "bad shape");
  if (M == 0) return TDP_OK;
  if (!logits || !out) return fail(TDP_EINVAL, "null pointer");
  HIP_TRY(launch_argmax_rows(logits, ld, M, n, out, (hipStream_t)stream));
  return TDP_OK;
}

}  // extern "C"
