// Bandwidth-trivial kernels of the stage: RMSNorm, rotary embedding fused with the KV-cache
// append, KV import/export, and the one-time weight repack.
//
// The KV cache (paper Sec. 2.1: per-token keys and values kept so that a decode step only
// processes the new token) is paged in fixed-size pages addressed through per-request block
// tables.  Physical layout per layer:
//   K pool  [num_pages][n_kv_heads][row bytes / 64][page_size][64 bytes]   (a key row in 64-byte pieces,
//           piece g of the page's 16 tokens together: what one decode-attention load instruction fetches
//           is then contiguous, see k_pool_byte)
//   V pool  [num_pages][n_kv_heads][head_dim][page_size]   (token index fastest)
// Keys are stored after rotation.  The V layout puts 8 consecutive tokens of one channel in
// 16 bytes, which is exactly the MFMA operand of the P*V product in both attention kernels.
#include "tdp_device.h"
#include "tdp_kernels.h"

namespace tdp {

// ------------------------------------------------------------------ RMSNorm
// y = x * g / sqrt(mean(x^2) + eps); one workgroup per row, fp32 statistics.  x is the residual
// stream: bf16 as handed over by the previous stage, fp32 between the layers of this stage.
template <bool F32_IN>
__device__ __forceinline__ void load8(const void* row, int c, float (&f)[8]) {
  if (F32_IN) {
    const f32x4 a = *reinterpret_cast<const f32x4*>((const float*)row + c * 8);
    const f32x4 b = *reinterpret_cast<const f32x4*>((const float*)row + c * 8 + 4);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[i] = a[i];
      f[i + 4] = b[i];
    }
  } else {
    const bf16x8 v = ld_bf16x8((const bf16*)row + c * 8);
#pragma unroll
    for (int i = 0; i < 8; ++i) f[i] = (float)v[i];
  }
}

template <bool F32_IN>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const void* __restrict__ x, int64_t ldx,
                                                      const float* __restrict__ gain, float eps, int d,
                                                      bf16* __restrict__ y, OperandLayout y_lay) {
  const int row = blockIdx.x;
  const void* xr = F32_IN ? (const void*)((const float*)x + (int64_t)row * ldx)
                          : (const void*)((const bf16*)x + (int64_t)row * ldx);
  const int chunks = d / 8;
  // the row is read once: a thread keeps its first KEEP chunks (a row of up to 8192 elements whole) in
  // registers between the two passes and re-reads only what lies beyond
  constexpr int KEEP = 4;
  float keep[KEEP][8];
  float ss = 0.f;
#pragma unroll
  for (int k = 0; k < KEEP; ++k) {
    const int c = threadIdx.x + 256 * k;
    if (c < chunks) {
      load8<F32_IN>(xr, c, keep[k]);
#pragma unroll
      for (int i = 0; i < 8; ++i) ss += keep[k][i] * keep[k][i];
    }
  }
  for (int c = threadIdx.x + 256 * KEEP; c < chunks; c += 256) {
    float f[8];
    load8<F32_IN>(xr, c, f);
#pragma unroll
    for (int i = 0; i < 8; ++i) ss += f[i] * f[i];
  }
  __shared__ float red[4];
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float tot = red[0] + red[1] + red[2] + red[3];
  const float inv = 1.0f / sqrtf(tot / (float)d + eps);
  auto emit = [&](int c, const float (&f)[8]) {
    const f32x4 g0 = *reinterpret_cast<const f32x4*>(gain + c * 8);
    const f32x4 g1 = *reinterpret_cast<const f32x4*>(gain + c * 8 + 4);
    bf16x8 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      o[i] = (bf16)(f[i] * inv * g0[i]);
      o[i + 4] = (bf16)(f[i + 4] * inv * g1[i]);
    }
    st_bf16x8(y + operand_offset(y_lay, row, c * 8), o);
  };
#pragma unroll
  for (int k = 0; k < KEEP; ++k) {
    const int c = threadIdx.x + 256 * k;
    if (c < chunks) emit(c, keep[k]);
  }
  for (int c = threadIdx.x + 256 * KEEP; c < chunks; c += 256) {
    float f[8];
    load8<F32_IN>(xr, c, f);
    emit(c, f);
  }
}

hipError_t launch_rmsnorm(const void* x, int x_is_f32, int64_t ldx, const float* gain, float eps, int M, int d,
                          void* y, OperandLayout y_layout, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  if (x_is_f32)
    rmsnorm_kernel<true><<<M, 256, 0, s>>>(x, ldx, gain, eps, d, (bf16*)y, y_layout);
  else
    rmsnorm_kernel<false><<<M, 256, 0, s>>>(x, ldx, gain, eps, d, (bf16*)y, y_layout);
  return hipGetLastError();
}

// Sum of split-K partials, eight consecutive columns at a time: acc = p_0 + p_1 + ... in split order
// (partial z of a row lies z * split_stride floats further on).  The partials are fetched UN
// splits at a time so that all of a thread's loads are in flight together: a loop that loads and adds
// one split per turn pays one memory round trip per split, which is what a launch of few rows
// (small decode batches) consists of.  `splits` is uniform, so the guards are scalar branches.
template <int NCOL, int UN>
__device__ __forceinline__ void sum_partials8(const float* const (&first)[NCOL], int64_t split_stride, int splits,
                                              float (&acc)[NCOL][8]) {
#pragma unroll
  for (int c = 0; c < NCOL; ++c)
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[c][i] = 0.f;
  for (int z0 = 0; z0 < splits; z0 += UN) {
    float f[UN][NCOL][8];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      if (z0 + u < splits) {
#pragma unroll
        for (int c = 0; c < NCOL; ++c) load8<true>(first[c] + (int64_t)(z0 + u) * split_stride, 0, f[u][c]);
      } else {
#pragma unroll
        for (int c = 0; c < NCOL; ++c)
#pragma unroll
          for (int i = 0; i < 8; ++i) f[u][c][i] = 0.f;
      }
    }
#pragma unroll
    for (int u = 0; u < UN; ++u)
#pragma unroll
      for (int c = 0; c < NCOL; ++c)
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[c][i] += f[u][c][i];
  }
}

// The row is formed first: h = residual + the split-K partials of the projection in front of the
// norm (summed in split order), stored as the fp32 residual stream, then normalised.  1024 threads
// per row: at d = 8192 every thread has one 8-element chunk, which it keeps in registers between the
// two passes; beyond that a thread re-reads what it wrote itself.
template <bool F32_RES>
__global__ __launch_bounds__(1024) void rmsnorm_sum_kernel(const void* __restrict__ residual, int64_t ldr,
                                                          const float* __restrict__ ws, int splits, int M,
                                                          int64_t ld_ws, float* __restrict__ h_out, int64_t ldh,
                                                          const float* __restrict__ gain, float eps, int d,
                                                          bf16* __restrict__ y, OperandLayout y_lay) {
  const int row = blockIdx.x;
  const void* rr = F32_RES ? (const void*)((const float*)residual + (int64_t)row * ldr)
                           : (const void*)((const bf16*)residual + (int64_t)row * ldr);
  float* hr = h_out + (int64_t)row * ldh;
  const int chunks = d / 8;
  const int64_t split_stride = (int64_t)M * ld_ws;
  float ss = 0.f;
  float keep[8];  // this thread's first chunk of h
  for (int c = threadIdx.x; c < chunks; c += 1024) {
    float f[8], acc[1][8];
    load8<F32_RES>(rr, c, f);
    const float* const first[1] = {ws + (int64_t)row * ld_ws + c * 8};
    sum_partials8<1, 8>(first, split_stride, splits, acc);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      acc[0][i] += f[i];
      ss += acc[0][i] * acc[0][i];
    }
    *reinterpret_cast<f32x4*>(hr + c * 8) = f32x4{acc[0][0], acc[0][1], acc[0][2], acc[0][3]};
    *reinterpret_cast<f32x4*>(hr + c * 8 + 4) = f32x4{acc[0][4], acc[0][5], acc[0][6], acc[0][7]};
    if (c == (int)threadIdx.x) {
#pragma unroll
      for (int i = 0; i < 8; ++i) keep[i] = acc[0][i];
    }
  }
  __shared__ float red[16];
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int w = 0; w < 16; ++w) tot += red[w];
  const float inv = 1.0f / sqrtf(tot / (float)d + eps);
  for (int c = threadIdx.x; c < chunks; c += 1024) {
    float f[8];
    if (c == (int)threadIdx.x) {
#pragma unroll
      for (int i = 0; i < 8; ++i) f[i] = keep[i];
    } else {
      load8<true>(hr, c, f);
    }
    const f32x4 g0 = *reinterpret_cast<const f32x4*>(gain + c * 8);
    const f32x4 g1 = *reinterpret_cast<const f32x4*>(gain + c * 8 + 4);
    bf16x8 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      o[i] = (bf16)(f[i] * inv * g0[i]);
      o[i + 4] = (bf16)(f[i + 4] * inv * g1[i]);
    }
    st_bf16x8(y + operand_offset(y_lay, row, c * 8), o);
  }
}

hipError_t launch_rmsnorm_sum(const void* residual, int residual_is_f32, int64_t ldr, const float* ws, int splits,
                              int64_t ld_ws, float* h_out, int64_t ldh, const float* gain, float eps, int M, int d,
                              void* y, OperandLayout y_layout, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  if (residual_is_f32)
    rmsnorm_sum_kernel<true><<<M, 1024, 0, s>>>(residual, ldr, ws, splits, M, ld_ws, h_out, ldh, gain, eps, d, (bf16*)y,
                                               y_layout);
  else
    rmsnorm_sum_kernel<false><<<M, 1024, 0, s>>>(residual, ldr, ws, splits, M, ld_ws, h_out, ldh, gain, eps, d,
                                                (bf16*)y, y_layout);
  return hipGetLastError();
}

// ------------------------------------------------------------------ token -> (sequence, position)
__device__ __forceinline__ void locate_token(int t, const int32_t* ctx_lens, const int32_t* cu_seqlens,
                                             int n_seqs, int& seq, int& pos) {
  if (ctx_lens) {  // decode: one token per request
    seq = t;
    pos = ctx_lens[t];
  } else {         // prefill: largest s with cu_seqlens[s] <= t
    int lo = 0, hi = n_seqs - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (cu_seqlens[mid] <= t) lo = mid; else hi = mid - 1;
    }
    seq = lo;
    pos = t - cu_seqlens[lo];
  }
}

// ------------------------------------------------------------------ RoPE + KV append
// One workgroup per token.  The projection arrives in fp32 - the GEMM's fp32 output, or its split-K
// partials, summed here in split order (plus the bias) - so the rotation works on unrounded sums and
// every query and key element is rounded exactly once, after the rotation.  q heads are rotated and
// written to the bf16 row the attention kernels read; k heads are rotated and written to the token's
// slot of the K pool; v heads are written (transposed) to the V pool, or, in prefill, rounded into
// the bf16 row for the page-by-page append that follows.  Rotation pairs channel i with channel
// i + head_dim/2 and turns the pair by pos * base^(-2i/head_dim); the table holds (cos, sin) of that
// angle, computed in double precision on the host.
template <int THREADS>
__global__ __launch_bounds__(THREADS) void rope_kv_kernel(bf16* __restrict__ qkv, int64_t ld, int n_q_heads,
                                                      KvLayout kv, const float2* __restrict__ table,
                                                      const int32_t* __restrict__ ctx_lens,
                                                      const int32_t* __restrict__ cu_seqlens, int n_seqs,
                                                      const int32_t* __restrict__ block_tables,
                                                      int max_pages_per_seq, const float* __restrict__ proj,
                                                      int splits, int n_tokens, const float* __restrict__ bias,
                                                      int v_to_row) {
  const int t = blockIdx.x;
  // NCOL groups of eight consecutive projection outputs of this token, starting at columns col[]
  const int64_t split_stride = (int64_t)n_tokens * ld;
  auto proj8 = [&](auto& f, auto... col) {
    constexpr int NCOL = sizeof...(col);
    const float* const first[NCOL] = {(proj + (int64_t)t * ld + col)...};
    const int cols[NCOL] = {col...};
    // one split per turn: fetching several at once costs registers, hence resident waves, and at the
    // batch sizes where this kernel takes measurable time (hundreds of rows) that loses more than it
    // gains (measured at batch 512: 23 us per launch against 21)
    sum_partials8<NCOL, 1>(first, split_stride, splits, f);
    if (bias) {
#pragma unroll
      for (int c = 0; c < NCOL; ++c) {
        float g[8];
        load8<true>(bias + cols[c], 0, g);
#pragma unroll
        for (int i = 0; i < 8; ++i) f[c][i] += g[i];
      }
    }
  };
  int seq, pos;
  locate_token(t, ctx_lens, cu_seqlens, n_seqs, seq, pos);
  const int dh = kv.head_dim, half = dh >> 1;
  const int page = block_tables[(int64_t)seq * max_pages_per_seq + pos / kv.page_size];
  const int slot = pos % kv.page_size;
  bf16* row = qkv + (int64_t)t * ld;
  const float2* cs = table + (int64_t)pos * half;
  const int per_head = half / 8;  // 16-byte units per half head
  const int rot_heads = n_q_heads + kv.n_kv_heads;
  bf16* vpool = (bf16*)kv.v_pool;
  for (int w = threadIdx.x; w < rot_heads * per_head; w += THREADS) {
    const int head = w / per_head;
    const int c0 = (w % per_head) * 8;
    bf16* hp = row + (int64_t)head * dh;
    float ab[2][8];
    proj8(ab, head * dh + c0, head * dh + half + c0);
    const float(&a)[8] = ab[0];
    const float(&b)[8] = ab[1];
    float fra[8], frb[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float2 t2 = cs[c0 + i];
      fra[i] = a[i] * t2.x - b[i] * t2.y;
      frb[i] = a[i] * t2.y + b[i] * t2.x;
    }
    // byte offsets of this thread's two 8-channel pieces in the K pool (a piece never straddles a 64-byte cut)
    const int esz = kv.fp8 ? 1 : 2;
    const int64_t k_lo = head >= n_q_heads ? k_pool_byte(kv, page, head - n_q_heads, slot, c0 * esz) : 0;
    const int64_t k_hi = head >= n_q_heads ? k_pool_byte(kv, page, head - n_q_heads, slot, (half + c0) * esz) : 0;
    if (head >= n_q_heads && kv.fp8) {
      // 8-bit cache: the rotated key goes from fp32 straight to its code (one rounding)
      uint2 ca = make_uint2(0u, 0u), cb = make_uint2(0u, 0u);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        ca.x |= f32_to_e4m3(fra[i] / kv.k_scale) << (8 * i);
        ca.y |= f32_to_e4m3(fra[4 + i] / kv.k_scale) << (8 * i);
        cb.x |= f32_to_e4m3(frb[i] / kv.k_scale) << (8 * i);
        cb.y |= f32_to_e4m3(frb[4 + i] / kv.k_scale) << (8 * i);
      }
      *reinterpret_cast<uint2*>((uint8_t*)kv.k_pool + k_lo) = ca;
      *reinterpret_cast<uint2*>((uint8_t*)kv.k_pool + k_hi) = cb;
      continue;
    }
    bf16x8 ra, rb;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      ra[i] = (bf16)fra[i];
      rb[i] = (bf16)frb[i];
    }
    if (head < n_q_heads) {
      st_bf16x8(hp + c0, ra);
      st_bf16x8(hp + half + c0, rb);
    } else {
      st_bf16x8(reinterpret_cast<bf16*>((uint8_t*)kv.k_pool + k_lo), ra);
      st_bf16x8(reinterpret_cast<bf16*>((uint8_t*)kv.k_pool + k_hi), rb);
    }
  }
  const int v_col = (n_q_heads + kv.n_kv_heads) * dh;
  for (int w8 = threadIdx.x; w8 < kv.n_kv_heads * dh / 8; w8 += THREADS) {
    float fv[1][8];
    proj8(fv, v_col + w8 * 8);
    const float(&f)[8] = fv[0];
    if (v_to_row) {  // prefill: the values are appended page by page (v_append_pages_kernel)
      bf16x8 o;
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] = (bf16)f[i];
      st_bf16x8(row + v_col + w8 * 8, o);
      continue;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int w = w8 * 8 + i;
      const int kvh = w / dh, c = w % dh;
      const int64_t vi = (((int64_t)page * kv.n_kv_heads + kvh) * dh + c) * kv.page_size + slot;
      // the value is a bf16 quantity in both forms of the cache (the 8-bit code is taken from it)
      const bf16 vb = (bf16)f[i];
      if (kv.fp8)
        ((uint8_t*)kv.v_pool)[vi] = (uint8_t)f32_to_e4m3((float)vb / kv.v_scale);
      else
        vpool[vi] = vb;
    }
  }
}

// Prefill, values rounded to bf16 in the token rows: the values of one page (up to 16 consecutive tokens of one
// prompt) are appended by one workgroup, so that a channel's row of the transposed V page is written
// as one piece (token by token every 2-byte store dirtied a 32-byte sector of its own: measured ten
// times the bytes).  Chunk w of the grid belongs to the last prompt s with cu_seqlens[s] / 16 + s <= w
// and is page w - (cu_seqlens[s] / 16 + s) of it; the numbering leaves every prompt room for all its
// pages, chunks past a prompt's last page do nothing.
__global__ __launch_bounds__(256) void v_append_pages_kernel(const bf16* __restrict__ qkv, int64_t ld, int v_col,
                                                             KvLayout kv, const int32_t* __restrict__ cu_seqlens,
                                                             int n_seqs, const int32_t* __restrict__ block_tables,
                                                             int max_pages_per_seq) {
  const int w = blockIdx.x;
  int lo = 0, hi = n_seqs - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if ((cu_seqlens[mid] >> 4) + mid <= w) lo = mid; else hi = mid - 1;
  }
  const int t_first = cu_seqlens[lo];
  const int len = cu_seqlens[lo + 1] - t_first;
  const int p = w - ((t_first >> 4) + lo);
  if (p < 0 || p * 16 >= len) return;
  const int n = min(16, len - p * 16);  // tokens on this page
  const int64_t page = block_tables[(int64_t)lo * max_pages_per_seq + p];
  const bf16* src = qkv + (int64_t)(t_first + p * 16) * ld + v_col;
  const int channels = kv.n_kv_heads * kv.head_dim;
  for (int c8 = threadIdx.x; c8 < channels / 8; c8 += 256) {
    bf16x8 in[16];  // [token][8 channels]
#pragma unroll
    for (int j = 0; j < 16; ++j) in[j] = j < n ? ld_bf16x8(src + (int64_t)j * ld + c8 * 8) : zero_bf16x8();
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      // pools are [page][kv head][channel][16 slots]: channel c8 * 8 + i of all kv heads, counted through
      const int64_t row = (page * channels + c8 * 8 + i) * 16;
      if (kv.fp8) {
        uint8_t* dst = (uint8_t*)kv.v_pool + row;
        uint4 codes = make_uint4(0u, 0u, 0u, 0u);
        uint32_t* cw = reinterpret_cast<uint32_t*>(&codes);
#pragma unroll
        for (int j = 0; j < 16; ++j) cw[j >> 2] |= f32_to_e4m3((float)in[j][i] / kv.v_scale) << (8 * (j & 3));
        if (n == 16) {
          *reinterpret_cast<uint4*>(dst) = codes;
        } else {
#pragma unroll
          for (int j = 0; j < 16; ++j)
            if (j < n) dst[j] = (uint8_t)(cw[j >> 2] >> (8 * (j & 3)));
        }
      } else {
        bf16* dst = (bf16*)kv.v_pool + row;
        bf16x8 a, b;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          a[j] = in[j][i];
          b[j] = in[8 + j][i];
        }
        if (n == 16) {
          st_bf16x8(dst, a);
          st_bf16x8(dst + 8, b);
        } else {
#pragma unroll
          for (int j = 0; j < 16; ++j)
            if (j < n) dst[j] = in[j][i];
        }
      }
    }
  }
}

hipError_t launch_rope_kv(void* qkv, int64_t ld, int n_tokens, int n_q_heads, const KvLayout& kv,
                          const float2* rope_table, int max_pos, const int32_t* ctx_lens,
                          const int32_t* cu_seqlens, int n_seqs, const int32_t* block_tables,
                          int max_pages_per_seq, const float* proj, int splits, const float* bias, hipStream_t s) {
  (void)max_pos;
  if (n_tokens <= 0) return hipSuccess;
  // prefill: the values go page by page; decode (one token per request) has nothing to gather
  const int paged_v = ctx_lens == nullptr;
  // with split-K partials to sum, 1024 threads per row keep all of a thread's loads in flight at once
  if (splits > 1)
    rope_kv_kernel<1024><<<n_tokens, 1024, 0, s>>>((bf16*)qkv, ld, n_q_heads, kv, rope_table, ctx_lens, cu_seqlens,
                                                  n_seqs, block_tables, max_pages_per_seq, proj, splits, n_tokens,
                                                  bias, paged_v);
  else
    rope_kv_kernel<256><<<n_tokens, 256, 0, s>>>((bf16*)qkv, ld, n_q_heads, kv, rope_table, ctx_lens, cu_seqlens,
                                                 n_seqs, block_tables, max_pages_per_seq, proj, 1, n_tokens, bias,
                                                 paged_v);
  if (paged_v)
    v_append_pages_kernel<<<(n_tokens >> 4) + n_seqs + 1, 256, 0, s>>>(
        (const bf16*)qkv, ld, (n_q_heads + kv.n_kv_heads) * kv.head_dim, kv, cu_seqlens, n_seqs, block_tables,
        max_pages_per_seq);
  return hipGetLastError();
}

// ------------------------------------------------------------------ KV import / export
__global__ __launch_bounds__(256) void kv_copy_kernel(int to_pages, bf16* __restrict__ k_packed,
                                                      bf16* __restrict__ v_packed, KvLayout kv,
                                                      const int32_t* __restrict__ cu_seqlens, int n_seqs,
                                                      const int32_t* __restrict__ block_tables,
                                                      int max_pages_per_seq) {
  const int t = blockIdx.x;
  int seq, pos;
  locate_token(t, nullptr, cu_seqlens, n_seqs, seq, pos);
  const int dh = kv.head_dim;
  const int page = block_tables[(int64_t)seq * max_pages_per_seq + pos / kv.page_size];
  const int slot = pos % kv.page_size;
  bf16* kpool = (bf16*)kv.k_pool;
  bf16* vpool = (bf16*)kv.v_pool;
  for (int w = threadIdx.x; w < kv.n_kv_heads * dh; w += 256) {
    const int kvh = w / dh, c = w % dh;
    const int64_t ki = k_pool_byte(kv, page, kvh, slot, c * (kv.fp8 ? 1 : 2)) / (kv.fp8 ? 1 : 2);  // element index
    const int64_t vi = (((int64_t)page * kv.n_kv_heads + kvh) * dh + c) * kv.page_size + slot;
    const int64_t pi = (int64_t)t * kv.n_kv_heads * dh + w;
    if (kv.fp8) {
      // packed side stays bf16: import encodes value / scale, export gives code value * scale
      uint8_t* k8 = (uint8_t*)kv.k_pool;
      uint8_t* v8 = (uint8_t*)kv.v_pool;
      if (to_pages) {
        k8[ki] = (uint8_t)f32_to_e4m3((float)k_packed[pi] / kv.k_scale);
        v8[vi] = (uint8_t)f32_to_e4m3((float)v_packed[pi] / kv.v_scale);
      } else {
        k_packed[pi] = (bf16)(e4m3_to_f32(k8[ki]) * kv.k_scale);
        v_packed[pi] = (bf16)(e4m3_to_f32(v8[vi]) * kv.v_scale);
      }
    } else if (to_pages) {
      kpool[ki] = k_packed[pi];
      vpool[vi] = v_packed[pi];
    } else {
      k_packed[pi] = kpool[ki];
      v_packed[pi] = vpool[vi];
    }
  }
}

// ------------------------------------------------------------------ E4M3 conversion (diagnostic)
__global__ void e4m3_encode_kernel(const float* __restrict__ src, uint8_t* __restrict__ dst, int64_t n, float scale) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = (uint8_t)f32_to_e4m3(src[i] / scale);
}
// decodes four codes per thread with the conversion the attention kernel uses; n is rounded up to
// a multiple of four by the caller's buffers
__global__ void e4m3_decode_kernel(const uint32_t* __restrict__ src, float* __restrict__ dst, int64_t n4) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n4) return;
  uint32_t lo, hi;
  e4m3x4_to_bf16x4(src[i], lo, hi);
  float4 o;
  o.x = __uint_as_float(lo << 16);
  o.y = __uint_as_float(lo & 0xffff0000u);
  o.z = __uint_as_float(hi << 16);
  o.w = __uint_as_float(hi & 0xffff0000u);
  reinterpret_cast<float4*>(dst)[i] = o;
}

hipError_t launch_e4m3_convert(int to_codes, const void* src, void* dst, int64_t n, float scale, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  if (to_codes)
    e4m3_encode_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>((const float*)src, (uint8_t*)dst, n, scale);
  else
    e4m3_decode_kernel<<<(unsigned)((n / 4 + 255) / 256), 256, 0, s>>>((const uint32_t*)src, (float*)dst, n / 4);
  return hipGetLastError();
}

hipError_t launch_kv_copy(int to_pages, void* k_packed, void* v_packed, const KvLayout& kv,
                          const int32_t* cu_seqlens, int n_seqs, int total_tokens,
                          const int32_t* block_tables, int max_pages_per_seq, hipStream_t s) {
  if (total_tokens <= 0) return hipSuccess;
  kv_copy_kernel<<<total_tokens, 256, 0, s>>>(to_pages, (bf16*)k_packed, (bf16*)v_packed, kv, cu_seqlens,
                                              n_seqs, block_tables, max_pages_per_seq);
  return hipGetLastError();
}

// ------------------------------------------------------------------ weight repack (one-time)
// dst(row_of(n), k) = bf16(src[k][n]) through a 32x32 LDS transpose; dst is in the weight layout
// (layout_weights) with dst_ld columns.
__global__ __launch_bounds__(256) void repack_kernel(const void* __restrict__ src, int src_is_f32,
                                                     int64_t K, int64_t N, int64_t ld_src, bf16* __restrict__ dst,
                                                     OperandLayout lay, int64_t row_off, int mode) {
  __shared__ float tile[32][33];
  const int64_t k0 = (int64_t)blockIdx.y * 32, n0 = (int64_t)blockIdx.x * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  for (int r = ty; r < 32; r += 8) {
    const int64_t k = k0 + r, n = n0 + tx;
    float v = 0.f;
    if (k < K && n < N)
      v = src_is_f32 ? ((const float*)src)[k * ld_src + n] : (float)((const bf16*)src)[k * ld_src + n];
    tile[r][tx] = v;
  }
  __syncthreads();
  for (int r = ty; r < 32; r += 8) {
    const int64_t n = n0 + r, k = k0 + tx;
    if (n < N && k < K) {
      int64_t row;
      if (mode == 0) row = row_off + n;
      else row = (n / 32) * 64 + (n % 32) + (mode == 2 ? 32 : 0);
      dst[operand_offset(lay, (int)row, (int)k)] = (bf16)tile[tx][r];
    }
  }
}

hipError_t launch_repack_ld(const void* src, int src_is_f32, int64_t rows_in, int64_t cols_out, int64_t ld_src,
                            void* dst, int64_t dst_ld, int64_t row_off, int mode, hipStream_t s) {
  dim3 grid((unsigned)((cols_out + 31) / 32), (unsigned)((rows_in + 31) / 32));
  repack_kernel<<<grid, 256, 0, s>>>(src, src_is_f32, rows_in, cols_out, ld_src, (bf16*)dst, layout_weights(dst_ld),
                                     row_off, mode);
  return hipGetLastError();
}

hipError_t launch_repack(const void* src, int src_is_f32, int64_t rows_in, int64_t cols_out, void* dst,
                         int64_t dst_ld, int64_t row_off, int mode, hipStream_t s) {
  return launch_repack_ld(src, src_is_f32, rows_in, cols_out, cols_out, dst, dst_ld, row_off, mode, s);
}

__global__ void convert_vec_kernel(const void* __restrict__ src, int src_is_f32, int64_t n,
                                   float* __restrict__ dst) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src_is_f32 ? ((const float*)src)[i] : (float)((const bf16*)src)[i];
}

hipError_t launch_convert_vec(const void* src, int src_is_f32, int64_t n, float* dst, hipStream_t s) {
  convert_vec_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(src, src_is_f32, n, dst);
  return hipGetLastError();
}

// ---- optional validation of device-side tables ---------------------------------------------
// The stage calls trust the tables they are given; these kernels are what a caller runs first when
// it does not.  They read a table only at (row < n, entry < max_pages_per_seq), whatever the lengths
// say, so they are safe on any input.  res[0] counts violations, res[1] keeps the smallest
// row * 8 + kind among them.
enum TableFault { kFaultLength = 1, kFaultPage = 2, kFaultShared = 3, kFaultPrefix = 4 };

__device__ __forceinline__ void table_fault(int32_t* res, int row, int kind) {
  atomicAdd(&res[0], 1);
  atomicMin(&res[1], row * 8 + kind);
}

__global__ void table_check_init_kernel(int32_t* __restrict__ owner, int num_pages, int32_t* __restrict__ res) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < num_pages) owner[i] = -1;
  if (i == 0) {
    res[0] = 0;
    res[1] = 0x7fffffff;
  }
}

// tokens of row r after the call (decode: ctx + 1; prefill: the prompt's length), or -1 if the
// length itself is invalid
__device__ __forceinline__ int table_row_tokens(int decode, const int32_t* lens, int r, int max_pos) {
  const int64_t n = decode ? (int64_t)lens[r] + 1 : (int64_t)lens[r + 1] - (int64_t)lens[r];
  const int64_t lo = decode ? 1 : 0;
  return (n < lo || n > max_pos) ? -1 : (int)n;
}

// pass 1: lengths, page ranges, and every page the call will WRITE is claimed by its row
// (decode: the page of position ctx; prefill: every page of the prompt)
__global__ __launch_bounds__(64) void table_check_claim_kernel(int decode, const int32_t* __restrict__ lens,
                                                               const int32_t* __restrict__ tables, int n_rows,
                                                               int max_pages_per_seq, int num_pages, int total_tokens,
                                                               int32_t* __restrict__ owner, int32_t* __restrict__ res) {
  const int r = blockIdx.x;
  if (!decode && r == 0 && threadIdx.x == 0) {
    if (lens[0] != 0) table_fault(res, 0, kFaultPrefix);
    if (lens[n_rows] != total_tokens) table_fault(res, n_rows - 1, kFaultPrefix);
  }
  const int n = table_row_tokens(decode, lens, r, max_pages_per_seq * 16);
  if (n < 0) {
    if (threadIdx.x == 0) table_fault(res, r, kFaultLength);
    return;
  }
  const int n_pages = (n + 15) / 16;
  for (int j = threadIdx.x; j < n_pages; j += 64) {
    const int p = tables[(int64_t)r * max_pages_per_seq + j];
    if (p < 0 || p >= num_pages) {
      table_fault(res, r, kFaultPage);
      continue;
    }
    if (!decode || j == n_pages - 1) {
      if (atomicCAS(&owner[p], -1, r) != -1) table_fault(res, r, kFaultShared);
    }
  }
}

// pass 2 (decode): no page that a row only reads is written by any row of the batch
__global__ __launch_bounds__(64) void table_check_read_kernel(const int32_t* __restrict__ lens,
                                                              const int32_t* __restrict__ tables,
                                                              int max_pages_per_seq, int num_pages,
                                                              const int32_t* __restrict__ owner,
                                                              int32_t* __restrict__ res) {
  const int r = blockIdx.x;
  const int n = table_row_tokens(1, lens, r, max_pages_per_seq * 16);
  if (n < 0) return;
  const int n_pages = (n + 15) / 16;
  for (int j = threadIdx.x; j < n_pages - 1; j += 64) {
    const int p = tables[(int64_t)r * max_pages_per_seq + j];
    if (p >= 0 && p < num_pages && owner[p] != -1) table_fault(res, r, kFaultShared);
  }
}

hipError_t launch_table_check(int decode, const int32_t* lens, const int32_t* tables, int n_rows,
                              int max_pages_per_seq, int num_pages, int total_tokens, int32_t* owner, int32_t* res,
                              hipStream_t s) {
  table_check_init_kernel<<<(num_pages + 255) / 256, 256, 0, s>>>(owner, num_pages, res);
  table_check_claim_kernel<<<n_rows, 64, 0, s>>>(decode, lens, tables, n_rows, max_pages_per_seq, num_pages,
                                                 total_tokens, owner, res);
  if (decode)
    table_check_read_kernel<<<n_rows, 64, 0, s>>>(lens, tables, max_pages_per_seq, num_pages, owner, res);
  return hipGetLastError();
}

// ---- pipeline ends: row gather (token embedding; last-token selection), bf16 conversion, argmax ----

// dst[m][:] = src[idx[m]][:]; one workgroup per row, 16-byte pieces.  An index outside
// [0, n_src_rows) is clamped into range, so a bad id can never read outside the table.
__global__ __launch_bounds__(256) void gather_rows_kernel(const bf16* __restrict__ src, int64_t ld_src,
                                                          int64_t n_src_rows, const int32_t* __restrict__ idx,
                                                          int d, bf16* __restrict__ dst, int64_t ld_dst) {
  const int m = blockIdx.x;
  int64_t r = idx[m];
  r = r < 0 ? 0 : (r >= n_src_rows ? n_src_rows - 1 : r);
  const bf16* sp = src + r * ld_src;
  bf16* dp = dst + (int64_t)m * ld_dst;
  for (int c = threadIdx.x * 8; c < d; c += 256 * 8) st_bf16x8(dp + c, ld_bf16x8(sp + c));
}

hipError_t launch_gather_rows(const void* src, int64_t ld_src, int64_t n_src_rows, const int32_t* idx, int M, int d,
                              void* dst, int64_t ld_dst, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  gather_rows_kernel<<<M, 256, 0, s>>>((const bf16*)src, ld_src, n_src_rows, idx, d, (bf16*)dst, ld_dst);
  return hipGetLastError();
}

__global__ void to_bf16_kernel(const void* __restrict__ src, int src_is_f32, int64_t n, bf16* __restrict__ dst) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src_is_f32 ? (bf16)((const float*)src)[i] : ((const bf16*)src)[i];
}

hipError_t launch_to_bf16(const void* src, int src_is_f32, int64_t n, void* dst, hipStream_t s) {
  to_bf16_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(src, src_is_f32, n, (bf16*)dst);
  return hipGetLastError();
}

// out[m] = the lowest index among the largest of logits[m][0 .. n).  One workgroup per row; a
// thread walks its columns in increasing order, so within a thread "strictly greater" keeps the
// first maximum, and the cross-thread reduction breaks value ties towards the lower index.
// NaNs never win a comparison; a row of NaNs gives 0.
__global__ __launch_bounds__(256) void argmax_rows_kernel(const float* __restrict__ logits, int64_t ld, int n,
                                                          int32_t* __restrict__ out) {
  __shared__ float s_val[256];
  __shared__ int s_idx[256];
  const float* row = logits + (int64_t)blockIdx.x * ld;
  float best = -INFINITY;
  int bi = 0x7fffffff;
  for (int j = threadIdx.x; j < n; j += 256) {
    const float v = row[j];
    if (v > best || (bi == 0x7fffffff && v == best)) {
      best = v;
      bi = j;
    }
  }
  s_val[threadIdx.x] = best;
  s_idx[threadIdx.x] = bi;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) {
      const float v = s_val[threadIdx.x + off];
      const int i = s_idx[threadIdx.x + off];
      if (v > s_val[threadIdx.x] || (v == s_val[threadIdx.x] && i < s_idx[threadIdx.x])) {
        s_val[threadIdx.x] = v;
        s_idx[threadIdx.x] = i;
      }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) out[blockIdx.x] = s_idx[0] == 0x7fffffff ? 0 : s_idx[0];
}

hipError_t launch_argmax_rows(const float* logits, int64_t ld, int M, int n, int32_t* out, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  argmax_rows_kernel<<<M, 256, 0, s>>>(logits, ld, n, out);
  return hipGetLastError();
}

}  // namespace tdp
