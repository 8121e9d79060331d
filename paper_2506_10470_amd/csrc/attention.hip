// Attention kernels of the stage: paged GQA decode attention (split over the KV range, then
// merged) and var-len causal prefill attention.  Both read K and V through the block tables.
//
// Decode (paper Sec. 2.1): each request contributes one query token that attends to its whole
// cache, so the kernel streams K/V once from HBM and is bandwidth bound.  The query heads that
// share a K/V head (GQA, Sec. 4.1) form the 16-wide "N" side of a 16x16x32 MFMA, so every K/V
// byte is loaded once per group and goes from global memory straight into MFMA operand
// registers: no LDS and no cross-lane transposes.
//
// The trick that avoids transposing the probabilities: scores are formed transposed,
// S^T[token][q] = K[token][:] . Q[q][:], and the rows of each MFMA tile are assigned to tokens in
// the order that makes a lane's accumulator elements the 8 consecutive tokens it must supply as
// the "B" operand of O^T[channel][q] += V^T[channel][token] P^T[token][q].
#include "tdp_device.h"
#include "tdp_kernels.h"

namespace tdp {

constexpr float kNegBig = -1.0e30f;  // finite stand-in for -inf: exp2 gives exactly 0, no inf-inf

// =====================================================================================
// Decode.  Work item = (request, span of span_len tokens of its context); one workgroup
// of four waves per (item, kv head).  The four waves split the span's 32-token blocks evenly and
// merge their partial softmax states through LDS; a request whose context fits one span is
// finished there (no partials in HBM), longer ones leave one partial per span for the merge
// kernel.  The item list is compact (built once per decode step by attn_plan_kernel), so the grid
// holds no workgroup that finds nothing to do except at its very end.
// Keys and values are requested as non-temporal: a launch reads each of them exactly once, and as
// ordinary loads they evict everything else from L2 on their way through (measured: 5.9 TB/s against
// 5.5 at batch 512, 5.7 against 5.2 at batch 256).
// =====================================================================================

// items[i] = (request, span index, tokens to attend to = ctx + 1, 0) for i < n_items[0], and
// (-1, ...) for the rest of the list up to max_items, so a workgroup learns everything about its
// work - or that it has none - from one 16-byte record.  One workgroup, any batch size.
// Longest work first: all full spans, then the requests' last (partial) spans by sixteenth of
// span_len, longest sixteenth first, so the workgroups that run at the end of the launch are short
// (with quarters the launch ended on workgroups of up to a quarter span in random order).
__global__ __launch_bounds__(256) void attn_plan_kernel(const int32_t* __restrict__ ctx_lens, int batch, int span_len,
                                                        int4* __restrict__ items, int max_items,
                                                        int32_t* __restrict__ n_items) {
  constexpr int NP = 16;      // parts of a span
  constexpr int NB = NP + 1;  // class 0: full spans; 1..NP: last span with > (NP-c)/NP of span_len
  __shared__ int part[NB][256];
  __shared__ int s_total;
  const int tid = threadIdx.x;
  const int per = (batch + 255) / 256;
  const int b0 = tid * per, b1 = min(b0 + per, batch);
  const int piece = span_len / NP;
  auto last_class = [&](int n_total, int n) {  // tokens in the last span: 1 .. span_len
    const int rem = n_total - (n - 1) * span_len;
    return NP - min((rem - 1) / piece, NP - 1);
  };
  for (int c = 0; c < NB; ++c) part[c][tid] = 0;
  for (int b = b0; b < b1; ++b) {
    const int n_total = ctx_lens[b] + 1;
    const int n = (n_total + span_len - 1) / span_len;
    part[0][tid] += n - 1;
    part[last_class(n_total, n)][tid] += 1;
  }
  __syncthreads();
  // exclusive prefix over (class, thread): thread c scans class c, then the class totals are chained
  __shared__ int class_total[NB];
  if (tid < NB) {
    int acc = 0;
    for (int i = 0; i < 256; ++i) {
      const int v = part[tid][i];
      part[tid][i] = acc;
      acc += v;
    }
    class_total[tid] = acc;
  }
  __syncthreads();
  if (tid == 0) {
    int acc = 0;
    for (int c = 0; c < NB; ++c) {
      const int v = class_total[c];
      class_total[c] = acc;
      acc += v;
    }
    n_items[0] = acc;
    s_total = acc;
  }
  __syncthreads();
  for (int c = 0; c < NB; ++c) part[c][tid] += class_total[c];
  for (int b = b0; b < b1; ++b) {
    const int n_total = ctx_lens[b] + 1;
    const int n = (n_total + span_len - 1) / span_len;
    for (int k = 0; k < n - 1; ++k) items[part[0][tid]++] = make_int4(b, k, n_total, 0);  // part[c][tid]: cursor
    items[part[last_class(n_total, n)][tid]++] = make_int4(b, n - 1, n_total, 0);
  }
  for (int i = s_total + tid; i < max_items; i += 256) items[i] = make_int4(-1, 0, 0, 0);
}

// item_pages[i][j] = physical page of the j-th 16-token page of item i's span (span_len / 16
// entries), entries past the request's last page clamped to it.  With this list a decode
// workgroup needs no look-up that depends on another look-up before its first K/V load.
__global__ __launch_bounds__(64) void attn_plan_pages_kernel(const int4* __restrict__ items,
                                                             const int32_t* __restrict__ block_tables,
                                                             int max_pages_per_seq, int pages_per_span,
                                                             int32_t* __restrict__ item_pages) {
  const int4 it = items[blockIdx.x];
  if (it.x < 0) return;
  const int last_page = (it.z - 1) / 16;
  for (int j = threadIdx.x; j < pages_per_span; j += 64) {
    const int p = min(it.y * pages_per_span + j, last_page);
    item_pages[(int64_t)blockIdx.x * pages_per_span + j] = block_tables[(int64_t)it.x * max_pages_per_seq + p];
  }
}

// KV8 = the pools hold E4M3 codes (one byte per element) instead of bf16.  A 16-byte load then carries
// 16 elements, which become two MFMA operands after conversion, so the block grows to 64 tokens
// (four pages) and the assignment of MFMA k-indices to channels (scores) and of score rows to
// tokens changes with it; the arithmetic after the conversion is the bf16 kernel's.  The cache
// scales ride along for free: k_scale in the softmax scale, v_scale in the final division.
template <int DH, bool KV8>
__global__ __launch_bounds__(256, 3) void attn_decode_kernel(const bf16* __restrict__ qkv, int64_t ld,
                                                          int n_q_heads, KvLayout kv,
                                                          const int4* __restrict__ items,
                                                          const int32_t* __restrict__ item_pages,
                                                          float* __restrict__ part_o, float* __restrict__ part_ml,
                                                          int max_spans, int span_len, bf16* __restrict__ out,
                                                          OperandLayout out_lay, float scale_log2, float out_scale) {
  constexpr int KS = DH / 32;          // k-steps of the score MFMA
  constexpr int DT = DH / 16;          // 16-channel tiles of the output
  constexpr int BT = KV8 ? 64 : 32;    // tokens per block
  constexpr int NT = BT / 16;          // score tiles per block
  constexpr int NP = BT / 32;          // k-steps of the output MFMA per block
  constexpr int LT = BT / 4;           // consecutive tokens of a block whose scores end up in one lane
  const int Hkv = kv.n_kv_heads;
  const int item = blockIdx.x / Hkv, kvh = blockIdx.x % Hkv;
  // the two look-ups a workgroup starts with are independent of each other: its work record and
  // its span's page list (lane j holds pages j, 64 + j, ...; at most 256 pages per span)
  const int pages_per_span = span_len >> 4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int my_pages[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
    my_pages[j] = item_pages[(int64_t)item * pages_per_span + min(lane + 64 * j, pages_per_span - 1)];
  const int4 it = items[item];
  if (it.x < 0) return;
  const int b = it.x, span = it.y;
  const int n_total = it.z;  // ctx + 1: the new token's K/V were appended before this kernel
  const int s_begin = span * span_len;
  const int s_end = min(s_begin + span_len, n_total);
  const int G = n_q_heads / Hkv;
  const int r16 = lane & 15, kg = lane >> 4;
  const bf16* kpool = (const bf16*)kv.k_pool;
  const bf16* vpool = (const bf16*)kv.v_pool;
  const uint8_t* kpool8 = (const uint8_t*)kv.k_pool;
  const uint8_t* vpool8 = (const uint8_t*)kv.v_pool;
  // this wave's share of the span, in whole blocks
  const int n_blocks = (s_end - s_begin + BT - 1) / BT;
  const int t_begin = s_begin + BT * ((wave * n_blocks) >> 2);
  const int t_end = min(s_begin + BT * (((wave + 1) * n_blocks) >> 2), s_end);

  // Query fragments.  bf16 pools: k-step kk covers channels kk*32 + kg*8 .. +8.  8-bit pools: a
  // lane's 16-byte key load covers channels ld*64 + kg*16 .. +16, whose halves feed k-steps 2 ld and
  // 2 ld + 1, so the query is gathered in that order.
  bf16x8 qf[KS];
  {
    const bf16* qp = qkv + (int64_t)b * ld + (int64_t)(kvh * G + (r16 < G ? r16 : 0)) * DH;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      const int ch = KV8 ? (kk >> 1) * 64 + kg * 16 + (kk & 1) * 8 : kk * 32 + kg * 8;
      qf[kk] = r16 < G ? ld_bf16x8(qp + ch) : zero_bf16x8();
    }
  }
  f32x4 o[DT];
#pragma unroll
  for (int d = 0; d < DT; ++d) o[d] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m = kNegBig, lsum = 0.f;

  if (t_begin < t_end) {
    // token (within its block) of this lane's row in score tile t: (r16/4)*LT + t*4 + r16%4; the
    // lane's own accumulator elements are then tokens kg*LT + t*4 + i, i.e. LT consecutive tokens
    const int krow0 = (r16 >> 2) * LT + (r16 & 3);
    // The span's page ids sit one per lane; the loop reads them with v_readlane, so no table load
    // sits between two blocks.  Entries past the request's last page were clamped to it by the
    // planner; pages of a span's last block that lie past the span are clamped to its last entry here.
    const int page_base = s_begin >> 4;

    // One block = the K fragments of NT score tiles and the V^T fragments of all channel tiles, 8 KiB
    // each per wave (head_dim 128).  K is fetched one block ahead into one of two register sets; V of
    // a block is fetched into a single set at the start of the block's own turn and is consumed
    // at its end, behind the score MFMAs and the softmax.  Per wave 16 KiB are in flight, and the
    // kernel fits three workgroups per CU (with both halves double-buffered it needed 198
    // registers, two workgroups per CU).  Measured: the same time either way (0.46-0.49 ms per
    // launch at batch 512, the spread coming from where the pools happen to lie in memory).
    struct KBlock {
      bf16x8 kf[2][KS];  // bf16 pools: [score tile][k-step]; 8-bit pools: 16 raw bytes per entry, [t / 2][(t % 2) * KS/2 + ld]
    };
    struct VBlock {
      bf16x8 vf[DT];     // bf16 pools: 8 tokens of a channel; 8-bit pools: 16 raw bytes = 16 tokens of a channel
    };
    auto page_of = [&](int i) -> int64_t {  // i is wave-uniform
      const int r = i >> 6;
      const int v = r == 0 ? my_pages[0] : r == 1 ? my_pages[1] : r == 2 ? my_pages[2] : my_pages[3];
      return __builtin_amdgcn_readlane(v, i & 63);
    };
    auto load_k = [&](int tb, KBlock& blk) {
      const int pi = (tb >> 4) - page_base;
      int64_t page[BT / 16];
#pragma unroll
      for (int j = 0; j < BT / 16; ++j) page[j] = page_of(min(pi + j, pages_per_span - 1));
      if constexpr (KV8) {
        // score tile t, row r16 -> token (r16/4)*16 + t*4 + r16%4: page r16/4 of the block, slot t*4 + r16%4
        const int64_t kpage = (r16 >> 2) == 0 ? page[0] : (r16 >> 2) == 1 ? page[1] : (r16 >> 2) == 2 ? page[2] : page[3];
        // (K pool: 64-byte pieces of the 16 token rows of a page lie together, piece l at l * 1024)
        const uint8_t* kp = kpool8 + (kpage * Hkv + kvh) * (16 * DH) + (r16 & 3) * 64 + kg * 16;
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
          for (int l = 0; l < KS / 2; ++l)
            blk.kf[t >> 1][(t & 1) * (KS / 2) + l] = ld_bf16x8_nt(reinterpret_cast<const bf16*>(kp + (t * 4) * 64 + l * 1024));
      } else {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const int tok = krow0 + t * 4;
          // (K pool: the 32 channels of k-step kk are one 64-byte piece; piece kk of the page's 16 tokens is
          // contiguous, so the 16 rows x 64 bytes of one instruction are four runs of 256 bytes)
          const bf16* kp = kpool + (page[tok >> 4 & 1] * Hkv + kvh) * (16 * DH) + (tok & 15) * 32 + kg * 8;
#pragma unroll
          for (int kk = 0; kk < KS; ++kk) blk.kf[t][kk] = ld_bf16x8_nt(kp + kk * (16 * 32));
        }
      }
    };
    auto load_v = [&](int tb, VBlock& blk) {
      const int pi = (tb >> 4) - page_base;
      int64_t page[BT / 16];  // the look-up index must be wave-uniform: all pages first, then the lane's pick
#pragma unroll
      for (int j = 0; j < BT / 16; ++j) page[j] = page_of(min(pi + j, pages_per_span - 1));
      if constexpr (KV8) {
        // channel r16 of tile d, the 16 tokens of page kg of the block
        const int64_t vpage = kg == 0 ? page[0] : kg == 1 ? page[1] : kg == 2 ? page[2] : page[3];
        const uint8_t* vp = vpool8 + ((vpage * Hkv + kvh) * DH + r16) * 16;
#pragma unroll
        for (int d = 0; d < DT; ++d) blk.vf[d] = ld_bf16x8_nt(reinterpret_cast<const bf16*>(vp + d * 16 * 16));
      } else {
        const int64_t vpage = kg < 2 ? page[0] : page[1];
        const bf16* vp = vpool + ((vpage * Hkv + kvh) * DH + r16) * 16 + (kg & 1) * 8;
#pragma unroll
        for (int d = 0; d < DT; ++d) blk.vf[d] = ld_bf16x8_nt(vp + d * 16 * 16);
      }
    };
    auto compute_block = [&](int tb, KBlock& blk, VBlock& vblk) {
      f32x4 s[NT];
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        s[t] = f32x4{0.f, 0.f, 0.f, 0.f};
        if constexpr (KV8) {
#pragma unroll
          for (int l = 0; l < KS / 2; ++l) {
            bf16x8 k0, k1;
            e4m3x16_to_bf16x8x2(__builtin_bit_cast(uint4, blk.kf[t >> 1][(t & 1) * (KS / 2) + l]), k0, k1);
            s[t] = mfma16(k0, qf[2 * l], s[t]);
            s[t] = mfma16(k1, qf[2 * l + 1], s[t]);
          }
        } else {
#pragma unroll
          for (int kk = 0; kk < KS; ++kk) s[t] = mfma16(blk.kf[t][kk], qf[kk], s[t]);
        }
      }
      // lane holds tokens tb + kg*LT + t*4 + i of column q = r16
      const int tok_base = tb + kg * LT;
      float mx = kNegBig;
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float v = (tok_base + t * 4 + i < n_total) ? s[t][i] * scale_log2 : kNegBig;
          s[t][i] = v;
          mx = fmaxf(mx, v);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m, mx);
      const float alpha = exp2f(m - m_new);
      bf16x8 pb[NP];
      float psum = 0.f;
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float pv = exp2f(s[t][i] - m_new);
          psum += pv;
          pb[t >> 1][(t & 1) * 4 + i] = (bf16)pv;
        }
      lsum = lsum * alpha + psum;
      m = m_new;
      const bool tail = tb + BT > n_total;  // slots past the context may hold anything, even NaN
#pragma unroll
      for (int d = 0; d < DT; ++d) {
        o[d] *= alpha;
        if constexpr (KV8) {
          uint4 raw = __builtin_bit_cast(uint4, vblk.vf[d]);
          if (tail) {  // keep the first n_total - tok_base bytes (tokens tok_base .. tok_base + 15)
            const int keep = min(max(n_total - tok_base, 0), 16);
            auto mask = [&](int w) -> uint32_t {
              const int k4 = min(max(keep - 4 * w, 0), 4);
              return k4 == 4 ? 0xffffffffu : (1u << (8 * k4)) - 1u;
            };
            raw.x &= mask(0);
            raw.y &= mask(1);
            raw.z &= mask(2);
            raw.w &= mask(3);
          }
          bf16x8 v0, v1;
          e4m3x16_to_bf16x8x2(raw, v0, v1);
          o[d] = mfma16(v0, pb[0], o[d]);
          o[d] = mfma16(v1, pb[NP - 1], o[d]);
        } else {
          if (tail) {
#pragma unroll
            for (int j = 0; j < 8; ++j)
              if (tok_base + j >= n_total) vblk.vf[d][j] = (bf16)0.0f;
          }
          o[d] = mfma16(vblk.vf[d], pb[0], o[d]);
        }
      }
    };

    // Two blocks per trip, K ping-pongs between two register sets.  Every block is loaded exactly
    // once: the steady-state loop only runs while two more blocks follow (its loads are
    // unconditional, so the compiler's wait counts stay exact), the last one or two blocks are
    // peeled off.
    KBlock k0, k1;
    VBlock v;
    int tb = t_begin;
    load_k(tb, k0);
    for (; tb + 2 * BT < t_end; tb += 2 * BT) {
      load_v(tb, v);
      load_k(tb + BT, k1);
      compute_block(tb, k0, v);
      load_v(tb + BT, v);
      load_k(tb + 2 * BT, k0);
      compute_block(tb + BT, k1, v);
    }
    if (tb + BT < t_end) {
      load_v(tb, v);
      load_k(tb + BT, k1);
      compute_block(tb, k0, v);
      load_v(tb + BT, v);
      compute_block(tb + BT, k1, v);
    } else {
      load_v(tb, v);
      compute_block(tb, k0, v);
    }
    lsum += __shfl_xor(lsum, 16, 64);
    lsum += __shfl_xor(lsum, 32, 64);
  }

  // ---- merge the four waves' states through LDS (fixed wave order: results do not depend on
  // which physical pages held the tokens)
  __shared__ float s_o[4][16][DH + 4];
  __shared__ float s_m[4][16], s_l[4][16];
#pragma unroll
  for (int d = 0; d < DT; ++d) *reinterpret_cast<f32x4*>(&s_o[wave][r16][d * 16 + kg * 4]) = o[d];
  if (kg == 0) {
    s_m[wave][r16] = m;
    s_l[wave][r16] = lsum;
  }
  __syncthreads();
  const int n_spans = (n_total + span_len - 1) / span_len;
  for (int e = threadIdx.x; e < G * DH; e += 256) {
    const int q = e / DH, c = e % DH;
    const float m0 = s_m[0][q], m1 = s_m[1][q], m2 = s_m[2][q], m3 = s_m[3][q];
    const float mt = fmaxf(fmaxf(m0, m1), fmaxf(m2, m3));
    const float w0 = exp2f(m0 - mt), w1 = exp2f(m1 - mt), w2 = exp2f(m2 - mt), w3 = exp2f(m3 - mt);
    const float num = w0 * s_o[0][q][c] + w1 * s_o[1][q][c] + w2 * s_o[2][q][c] + w3 * s_o[3][q][c];
    const float den = w0 * s_l[0][q] + w1 * s_l[1][q] + w2 * s_l[2][q] + w3 * s_l[3][q];
    const int h = kvh * G + q;
    if (n_spans == 1) {
      out[operand_offset(out_lay, b, h * DH + c)] = (bf16)(num / den * out_scale);
    } else {
      const int64_t slot = ((int64_t)b * n_q_heads + h) * max_spans + span;
      part_o[slot * DH + c] = num;
      if (c == 0) {
        part_ml[slot * 2 + 0] = mt;
        part_ml[slot * 2 + 1] = den;
      }
    }
  }
}

// Requests longer than one span: out = sum_s o_s 2^(m_s - m) / sum_s l_s 2^(m_s - m).
template <int DH>
__global__ __launch_bounds__(DH) void attn_decode_merge_kernel(const float* __restrict__ part_o,
                                                               const float* __restrict__ part_ml,
                                                               const int32_t* __restrict__ ctx_lens,
                                                               int n_q_heads, int max_spans, int span_len,
                                                               bf16* __restrict__ out, OperandLayout out_lay,
                                                               float out_scale) {
  const int h = blockIdx.x, b = blockIdx.y, c = threadIdx.x;
  const int n_spans = min((ctx_lens[b] + span_len) / span_len, max_spans);
  if (n_spans <= 1) return;  // finished by the attention kernel itself
  const int64_t base = ((int64_t)b * n_q_heads + h) * max_spans;
  float m = kNegBig;
  for (int k = 0; k < n_spans; ++k) m = fmaxf(m, part_ml[(base + k) * 2]);
  float num = 0.f, den = 0.f;
  for (int k = 0; k < n_spans; ++k) {
    const float w = exp2f(part_ml[(base + k) * 2] - m);
    den += w * part_ml[(base + k) * 2 + 1];
    num += w * part_o[(base + k) * DH + c];
  }
  out[operand_offset(out_lay, b, h * DH + c)] = (bf16)(num / den * out_scale);
}

// Span length.  A workgroup's fixed costs (start-up, the merge of its four waves, its partial
// result) are paid once per span, so spans should be as long as the batch allows while the launch
// still has several workgroups per CU; a context that fits one span needs no partials at all.
// Measured on the 70B shape (attention ms per layer at spans 256 / 1024 / 2048 / 4096): batch 16:
// .032 / .028 / .035 / .046; batch 128: .158 / .138 / .137 / .138; batch 512: .610 / .521 / .494 / .487.
int attn_decode_span(int batch, int n_kv_heads) {
  const int units = batch * n_kv_heads;
  return units >= 4096 ? 4096 : units >= 1024 ? 2048 : units >= 128 ? 1024 : kDecodeSpanMin;
}

int attn_decode_items(int batch, int max_spans, int span_len) {
  // max_spans counts spans of the minimum length; longer spans need proportionally fewer slots
  return batch * ((max_spans * kDecodeSpanMin + span_len - 1) / span_len);
}

hipError_t launch_attn_plan(const int32_t* ctx_lens, const int32_t* block_tables, int max_pages_per_seq, int batch,
                            int max_spans, int span_len, int4* items, int32_t* n_items, int32_t* item_pages,
                            hipStream_t s) {
  if (batch <= 0) return hipSuccess;
  const int max_items = attn_decode_items(batch, max_spans, span_len);
  attn_plan_kernel<<<1, 256, 0, s>>>(ctx_lens, batch, span_len, items, max_items, n_items);
  attn_plan_pages_kernel<<<max_items, 64, 0, s>>>(items, block_tables, max_pages_per_seq, span_len / 16, item_pages);
  return hipGetLastError();
}

hipError_t launch_attn_decode(const void* qkv, int64_t ld, int batch, int n_q_heads, const KvLayout& kv,
                              const int4* items, const int32_t* item_pages, float* part_o, float* part_ml,
                              int max_spans, int span_len, void* out, OperandLayout out_layout, hipStream_t s) {
  if (batch <= 0) return hipSuccess;
  // 8-bit pools hold value / scale: the key scale joins the softmax scale, the value scale the final division
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)kv.head_dim) * (kv.fp8 ? kv.k_scale : 1.0f);
  const float out_scale = kv.fp8 ? kv.v_scale : 1.0f;
  const int max_items = attn_decode_items(batch, max_spans, span_len);
  const unsigned grid = (unsigned)max_items * kv.n_kv_heads;
#define TDP_DECODE(DH, KV8)                                                                                        \
  attn_decode_kernel<DH, KV8><<<grid, 256, 0, s>>>((const bf16*)qkv, ld, n_q_heads, kv, items, item_pages, part_o, \
                                                   part_ml, max_spans, span_len, (bf16*)out, out_layout,          \
                                                   scale_log2, out_scale)
  if (kv.head_dim == 128) {
    if (kv.fp8) TDP_DECODE(128, true); else TDP_DECODE(128, false);
  } else {
    if (kv.fp8) TDP_DECODE(64, true); else TDP_DECODE(64, false);
  }
#undef TDP_DECODE
  return hipGetLastError();
}

hipError_t launch_attn_decode_merge(int batch, int n_q_heads, const KvLayout& kv, const int32_t* ctx_lens,
                                    const float* part_o, const float* part_ml, int max_spans, int span_len, void* out,
                                    OperandLayout out_layout, hipStream_t s) {
  if (batch <= 0) return hipSuccess;
  // with one span per request at most, every request was finished by the attention kernel itself
  if (attn_decode_items(batch, max_spans, span_len) / batch <= 1) return hipSuccess;
  const float out_scale = kv.fp8 ? kv.v_scale : 1.0f;
  dim3 mgrid(n_q_heads, batch);
  if (kv.head_dim == 128)
    attn_decode_merge_kernel<128><<<mgrid, 128, 0, s>>>(part_o, part_ml, ctx_lens, n_q_heads, max_spans, span_len,
                                                        (bf16*)out, out_layout, out_scale);
  else
    attn_decode_merge_kernel<64><<<mgrid, 64, 0, s>>>(part_o, part_ml, ctx_lens, n_q_heads, max_spans, span_len,
                                                      (bf16*)out, out_layout, out_scale);
  return hipGetLastError();
}

// =====================================================================================
// Prefill: var-len packed, causal.  One workgroup of eight waves per tile of 256 query columns that
// share one K/V head: NH query heads of a GQA group x 256/NH consecutive positions (NH = 1 for
// multi-head attention: 256 positions of one head); each wave owns 32 columns.  Each 32-token
// block of K and V^T is staged once per workgroup in LDS (double buffered, XOR-swizzled against
// bank conflicts) and feeds the MFMAs of all 256 columns, so K/V traffic per MFMA is 1/8 of a
// wave-private scheme.  Two waves share a SIMD, so one wave's softmax arithmetic overlaps the
// other's MFMAs; the softmax itself is trimmed to what a wave64 vector unit can keep up with:
// one FMA + one raw exp2 per score, masking only in blocks that cross the diagonal or the end of
// the prompt, and the running maximum is only raised (and the accumulator rescaled) when a
// block's maximum exceeds it by more than 2^8, which keeps every probability below 256.
// Same transposed-score trick as decode: S^T = K Q^T with score rows permuted so that a lane's
// accumulator elements are the 8 consecutive tokens it supplies to O^T += V^T P^T.
// =====================================================================================
constexpr float kRescaleSlack = 8.0f;  // log2 units

// KV8: the pools hold E4M3 codes; a thread's chunk is then 8 bytes, converted to bf16 on its way into
// LDS (the key scale rides in the softmax scale, the value scale in the final normalisation).
template <int DH, int NH, bool KV8>
__global__ __launch_bounds__(512) void attn_prefill_kernel(const bf16* __restrict__ qkv, int64_t ld,
                                                           int n_q_heads, KvLayout kv,
                                                           const int32_t* __restrict__ cu_seqlens, int n_seqs,
                                                           const int32_t* __restrict__ block_tables,
                                                           int max_pages_per_seq, bf16* __restrict__ out,
                                                           OperandLayout out_lay, float scale_log2, float out_scale) {
  constexpr int NP = 256 / NH;   // query positions per workgroup
  constexpr int PB = NP / 32;    // 32-position blocks per head
  constexpr int KS = DH / 16;    // k-steps of the score MFMA
  constexpr int DT = DH / 32;    // 32-channel tiles of the output
  constexpr int CR = DH / 8;     // 16-byte chunks per K row
  constexpr int RWK = DH == 128 ? 1 : 2;  // K rows per 256-byte bank window
  constexpr int NCH = CR / 8;    // chunks of K, and of V^T, per thread per 64-token block
  constexpr int QP = KV8 ? 8 : 4;  // 8-element chunks per 64-byte piece of a key row in the pool
  __shared__ __attribute__((aligned(16))) bf16 sK[2][2][32 * DH];  // [buffer][32-token half]
  __shared__ __attribute__((aligned(16))) bf16 sV[2][2][DH * 32];

  // locate the sequence that owns query tile blockIdx.x
  int qt = blockIdx.x, s = 0, L = 0;
  for (; s < n_seqs; ++s) {
    L = cu_seqlens[s + 1] - cu_seqlens[s];
    const int nt = (L + NP - 1) / NP;
    if (qt < nt) break;
    qt -= nt;
  }
  if (s == n_seqs) return;
  const int tok0 = cu_seqlens[s];
  const int q0 = qt * NP;
  const int Hkv = kv.n_kv_heads;
  const int G = n_q_heads / Hkv;
  const int groups = G / NH;
  const int kvh = blockIdx.y / groups;
  const int h_base = kvh * G + (blockIdx.y % groups) * NH;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, kg = lane >> 5;
  const bf16* kpool = (const bf16*)kv.k_pool;
  const bf16* vpool = (const bf16*)kv.v_pool;

  // the wave's 32 query columns: one head, 32 consecutive positions
  const int head = h_base + wave / PB;
  const int p_first = q0 + (wave % PB) * 32;
  const int qpos = p_first + l32;  // may lie past the end of the prompt: computed, never stored
  const int p_last = min(p_first + 31, L - 1);
  bf16x8 qf[KS];
  {
    const bf16* qp = qkv + (int64_t)(tok0 + min(qpos, L - 1)) * ld + (int64_t)head * DH + kg * 8;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) qf[kk] = ld_bf16x8(qp + kk * 16);
  }
  f32x16 o[DT];
#pragma unroll
  for (int d = 0; d < DT; ++d)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[d][i] = 0.f;
  float m = kNegBig, lsum = 0.f;

  const int32_t* bt = block_tables + (int64_t)s * max_pages_per_seq;
  const int last_page = (L - 1) / 16;
  const int kv_end = min(q0 + NP, L);
  // token of this lane's row r = l32 in the score tile: (r/16)*16 + ((r%8)/4)*8 + ((r/8)%2)*4 + r%4
  const int krow = (l32 >> 4) * 16 + ((l32 >> 2) & 1) * 8 + ((l32 >> 3) & 1) * 4 + (l32 & 3);
  const bf16* k_frag = &sK[0][0][0] + krow * DH;
  const int k_swz = (krow / RWK) % CR;

  // staging: this thread's chunks of K and of V^T of the next 64-token block (two 32-token halves)
  bf16x8 kreg[NCH], vreg[NCH];
  auto load_block = [&](int kb) {
    const int p0 = kb >> 4;
    int64_t page[4];  // never dereference a table entry past the last page
#pragma unroll
    for (int i = 0; i < 4; ++i) page[i] = bt[min(p0 + i, last_page)];
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      const int ci = tid + 512 * j;
      // K: consecutive threads walk the pool in address order - the QP chunks of a 64-byte piece, the 16
      // tokens of the page, the pieces of the row, the four pages of the block
      const int kq = ci % QP, kt16 = (ci / QP) % 16, kpiece = (ci / (QP * 16)) % (CR / QP), kpg = ci / (16 * CR);
      const int64_t kp = page[kpg];
      const int vsub = ci / (DH * 4), vr = (ci >> 2) % DH, vc = ci & 3;
      const int64_t vp = vsub ? (vc < 2 ? page[2] : page[3]) : (vc < 2 ? page[0] : page[1]);
      const int64_t k_at = (kp * Hkv + kvh) * (16 * DH) + (kpiece * 16 + kt16) * (QP * 8) + kq * 8;
      const int64_t v_at = ((vp * Hkv + kvh) * DH + vr) * 16 + (vc & 1) * 8;
      bf16x8 v;
      if constexpr (KV8) {
        union {
          uint32_t u[4];
          bf16x8 x;
        } ck, cv;
        const uint2 rk = *reinterpret_cast<const uint2*>((const uint8_t*)kv.k_pool + k_at);
        const uint2 rv = *reinterpret_cast<const uint2*>((const uint8_t*)kv.v_pool + v_at);
        e4m3x4_to_bf16x4(rk.x, ck.u[0], ck.u[1]);
        e4m3x4_to_bf16x4(rk.y, ck.u[2], ck.u[3]);
        e4m3x4_to_bf16x4(rv.x, cv.u[0], cv.u[1]);
        e4m3x4_to_bf16x4(rv.y, cv.u[2], cv.u[3]);
        kreg[j] = ck.x;
        v = cv.x;
      } else {
        kreg[j] = ld_bf16x8(kpool + k_at);
        v = ld_bf16x8(vpool + v_at);
      }
      if (kb + 64 > L) {  // slots past the prompt may hold anything, even NaN
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (kb + vsub * 32 + vc * 8 + e >= L) v[e] = (bf16)0.0f;
      }
      vreg[j] = v;
    }
  };
  auto store_block = [&](int buf) {
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      const int ci = tid + 512 * j;
      const int kq = ci % QP, kt16 = (ci / QP) % 16, kpiece = (ci / (QP * 16)) % (CR / QP), kpg = ci / (16 * CR);
      const int ksub = kpg >> 1, ktok = (kpg & 1) * 16 + kt16, kc = kpiece * QP + kq;
      st_bf16x8(&sK[buf][ksub][ktok * DH + ((kc ^ ((ktok / RWK) % CR)) << 3)], kreg[j]);
      const int vsub = ci / (DH * 4), vr = (ci >> 2) % DH, vc = ci & 3;
      st_bf16x8(&sV[buf][vsub][vr * 32 + ((vc ^ ((vr >> 2) & 3)) << 3)], vreg[j]);
    }
  };

  load_block(0);
  store_block(0);
  __syncthreads();
  for (int kb0 = 0, buf = 0; kb0 < kv_end; kb0 += 64, buf ^= 1) {
    const bool more = kb0 + 64 < kv_end;
    if (more) load_block(kb0 + 64);
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      const int kb = kb0 + sub * 32;
      // causal: blocks past the wave's last row contribute nothing
      if (kb > p_last || p_first >= L) continue;
      f32x16 sc;
#pragma unroll
      for (int i = 0; i < 16; ++i) sc[i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KS; ++kk)
        sc = mfma32(ld_bf16x8(k_frag + (buf * 2 + sub) * 32 * DH + (((kk * 2 + kg) ^ k_swz) << 3)), qf[kk], sc);
      // element i of this lane is token kb + (i/8)*16 + kg*8 + i%8 of query column qpos
      if (kb + 31 > p_first || kb + 32 > L) {  // the block crosses the diagonal or the prompt's end
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int tok = kb + (i >> 3) * 16 + kg * 8 + (i & 7);
          if (!(tok <= qpos && tok < L)) sc[i] = kNegBig;
        }
      }
      float mx = sc[0];
#pragma unroll
      for (int i = 1; i < 16; ++i) mx = fmaxf(mx, sc[i]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * scale_log2;  // scale > 0: max commutes with it
      if (__any(mx > m + kRescaleSlack)) {
        const float m_new = fmaxf(m, mx);
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        lsum *= alpha;
        m = m_new;
#pragma unroll
        for (int d = 0; d < DT; ++d)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[d][i] *= alpha;
      }
      bf16x8 pb[2];
      float psum = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float pv = __builtin_amdgcn_exp2f(fmaf(sc[i], scale_log2, -m));
        psum += pv;
        pb[i >> 3][i & 7] = (bf16)pv;
      }
      lsum += psum;
#pragma unroll
      for (int d = 0; d < DT; ++d) {
        const int r = d * 32 + l32;
#pragma unroll
        for (int st = 0; st < 2; ++st)
          o[d] = mfma32(ld_bf16x8(&sV[buf][sub][r * 32 + (((st * 2 + kg) ^ ((r >> 2) & 3)) << 3)]), pb[st], o[d]);
      }
    }
    if (more) store_block(buf ^ 1);
    __syncthreads();
  }
  lsum += __shfl_xor(lsum, 32, 64);
  if (qpos < L) {
    const float inv = out_scale / lsum;
#pragma unroll
    for (int d = 0; d < DT; ++d)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (bf16)(o[d][g * 4 + e] * inv);
        *reinterpret_cast<bf16x4*>(out + operand_offset(out_lay, tok0 + qpos, head * DH + d * 32 + g * 8 + kg * 4)) =
            v;
      }
  }
}

template <int DH, int NH>
static hipError_t launch_attn_prefill_t(const void* qkv, int64_t ld, int total_tokens, int n_seqs, int n_q_heads,
                                        const KvLayout& kv, const int32_t* cu_seqlens, const int32_t* block_tables,
                                        int max_pages_per_seq, void* out, OperandLayout out_layout, hipStream_t s) {
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)kv.head_dim) * (kv.fp8 ? kv.k_scale : 1.0f);
  const float out_scale = kv.fp8 ? kv.v_scale : 1.0f;
  constexpr int NP = 256 / NH;
  dim3 grid((total_tokens + NP - 1) / NP + n_seqs, n_q_heads / NH);
  if (kv.fp8)
    attn_prefill_kernel<DH, NH, true><<<grid, 512, 0, s>>>((const bf16*)qkv, ld, n_q_heads, kv, cu_seqlens, n_seqs,
                                                           block_tables, max_pages_per_seq, (bf16*)out, out_layout,
                                                           scale_log2, out_scale);
  else
    attn_prefill_kernel<DH, NH, false><<<grid, 512, 0, s>>>((const bf16*)qkv, ld, n_q_heads, kv, cu_seqlens, n_seqs,
                                                            block_tables, max_pages_per_seq, (bf16*)out, out_layout,
                                                            scale_log2, out_scale);
  return hipGetLastError();
}

hipError_t launch_attn_prefill(const void* qkv, int64_t ld, int total_tokens, int n_seqs, int n_q_heads,
                               const KvLayout& kv, const int32_t* cu_seqlens, const int32_t* block_tables,
                               int max_pages_per_seq, void* out, OperandLayout out_layout, hipStream_t s) {
  if (total_tokens <= 0 || n_seqs <= 0) return hipSuccess;
  const int G = n_q_heads / kv.n_kv_heads;
  const int nh = G % 8 == 0 ? 8 : G % 4 == 0 ? 4 : G % 2 == 0 ? 2 : 1;
#define TDP_PREFILL(DH_, NH_)                                                                               \
  return launch_attn_prefill_t<DH_, NH_>(qkv, ld, total_tokens, n_seqs, n_q_heads, kv, cu_seqlens, block_tables, \
                                         max_pages_per_seq, out, out_layout, s)
  if (kv.head_dim == 128) {
    if (nh == 8) TDP_PREFILL(128, 8);
    if (nh == 4) TDP_PREFILL(128, 4);
    if (nh == 2) TDP_PREFILL(128, 2);
    TDP_PREFILL(128, 1);
  } else {
    if (nh == 8) TDP_PREFILL(64, 8);
    if (nh == 4) TDP_PREFILL(64, 4);
    if (nh == 2) TDP_PREFILL(64, 2);
    TDP_PREFILL(64, 1);
  }
#undef TDP_PREFILL
}

}  // namespace tdp
