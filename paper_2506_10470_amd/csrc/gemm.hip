// bf16 MFMA GEMM for the stage's four projections (paper Sec. 3.4: linear layers dominate the
// execution time of a decode step, and only the batch size sets their cost).
//
//   out[M, N] = epilogue( A[M, K] * W^T ),   A bf16 [M][lda],  W bf16 [Npad][Kpad]  (K contiguous)
//
// Both operands are K-contiguous, so an MFMA fragment is one 16-byte load.  The product is formed
// transposed, D[n][m] = sum_k W[n][k] A[m][k], with the weights as the MFMA "A" operand: a lane
// then holds four consecutive output columns n of one row m, which makes the epilogue's stores
// 8 bytes wide and lets the SwiGLU epilogue find gate and up of one column in the same lane.
//
// Tiles are staged through LDS (double buffered, one barrier per 64-wide k-tile) with an XOR
// swizzle of the 16-byte chunks so that both the staging writes and the fragment reads are free
// of bank conflicts.  For small M (decode) the K range is split across workgroups and fp32
// partials are reduced by a second kernel that applies the epilogue.
#include "tdp_device.h"
#include "tdp_kernels.h"

namespace tdp {

struct GemmParams {
  const bf16* A;
  const bf16* W;
  bf16* out;
  const bf16* residual;
  float* ws;
  int64_t lda, Kpad, Npad, ldo, ldr;
  int M, N_store, epilogue;
  int k_tiles_total, k_tiles_per_split, splits;
  int tiles_m, tiles_n;
};

__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

template <int BM, int BN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(256) void gemm_kernel(const GemmParams p) {
  constexpr int BK = 64;
  constexpr int TM = BM / WAVES_M / 32;
  constexpr int TN = BN / WAVES_N / 32;
  static_assert(WAVES_M * WAVES_N == 4, "four waves per workgroup");
  static_assert(TN % 2 == 0, "gate/up pairing needs an even number of 32-row weight tiles per wave");
  constexpr int A_LOADS = BM / 32;  // 16-byte chunks per thread per k-tile
  constexpr int W_LOADS = BN / 32;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16* sA = reinterpret_cast<bf16*>(smem_raw);          // [2][BM][64]
  bf16* sW = sA + 2 * BM * BK;                           // [2][BN][64]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm0 = (wave / WAVES_N) * (TM * 32);
  const int wn0 = (wave % WAVES_N) * (TN * 32);
  const int l32 = lane & 31;
  const int kg = lane >> 5;

  const int tile = blockIdx.x;
  const int tile_n = tile % p.tiles_n;
  const int tile_m = tile / p.tiles_n;
  const int split = blockIdx.y;
  const int m0 = tile_m * BM;
  const int n0 = tile_n * BN;
  const int kt_begin = split * p.k_tiles_per_split;
  int kt_end = kt_begin + p.k_tiles_per_split;
  if (kt_end > p.k_tiles_total) kt_end = p.k_tiles_total;

  // staging assignment: thread -> (row = tid/8 + 32 j, chunk = tid%8)
  const int ld_row = tid >> 3;
  const int ld_chunk = tid & 7;
  const bf16* a_ptr[A_LOADS];
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) {
    int m = m0 + ld_row + 32 * j;
    if (m > p.M - 1) m = p.M - 1;  // rows past M are clamped: computed, never stored
    a_ptr[j] = p.A + (int64_t)m * p.lda + ld_chunk * 8;
  }
  const bf16* w_ptr = p.W + (int64_t)(n0 + ld_row) * p.Kpad + ld_chunk * 8;

  bf16x8 a_reg[A_LOADS], w_reg[W_LOADS];
  auto load_global = [&](int kt) {
    const int64_t k = (int64_t)kt * BK;
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j) a_reg[j] = ld_bf16x8(a_ptr[j] + k);
#pragma unroll
    for (int j = 0; j < W_LOADS; ++j) w_reg[j] = ld_bf16x8(w_ptr + (int64_t)(32 * j) * p.Kpad + k);
  };
  auto store_lds = [&](int buf) {
    bf16* a = sA + buf * BM * BK;
    bf16* w = sW + buf * BN * BK;
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j) {
      const int r = ld_row + 32 * j;
      st_bf16x8(a + r * BK + ((ld_chunk ^ (r & 7)) << 3), a_reg[j]);
    }
#pragma unroll
    for (int j = 0; j < W_LOADS; ++j) {
      const int r = ld_row + 32 * j;
      st_bf16x8(w + r * BK + ((ld_chunk ^ (r & 7)) << 3), w_reg[j]);
    }
  };

  f32x16 acc[TN][TM];
#pragma unroll
  for (int tn = 0; tn < TN; ++tn)
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[tn][tm][i] = 0.0f;

  if (kt_begin < kt_end) {
    load_global(kt_begin);
    store_lds(0);
  }
  __syncthreads();

  for (int kt = kt_begin; kt < kt_end; ++kt) {
    const int buf = (kt - kt_begin) & 1;
    const bool more = kt + 1 < kt_end;
    if (more) load_global(kt + 1);
    const bf16* a = sA + buf * BM * BK;
    const bf16* w = sW + buf * BN * BK;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int chunk = kk * 2 + kg;
      bf16x8 wf[TN], af[TM];
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) {
        const int r = wn0 + tn * 32 + l32;
        wf[tn] = ld_bf16x8(w + r * BK + ((chunk ^ (r & 7)) << 3));
      }
#pragma unroll
      for (int tm = 0; tm < TM; ++tm) {
        const int r = wm0 + tm * 32 + l32;
        af[tm] = ld_bf16x8(a + r * BK + ((chunk ^ (r & 7)) << 3));
      }
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) acc[tn][tm] = mfma32(wf[tn], af[tm], acc[tn][tm]);
    }
    if (more) store_lds(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: lane holds, for each (tn, tm, g), columns n..n+3 of row m -------------------
#pragma unroll
  for (int tm = 0; tm < TM; ++tm) {
    const int m = m0 + wm0 + tm * 32 + l32;
    if (m >= p.M) continue;
    if (p.splits > 1) {
      float* dst = p.ws + ((int64_t)split * p.M + m) * p.Npad;
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int n = n0 + wn0 + tn * 32 + g * 8 + kg * 4;
          f32x4 v = {acc[tn][tm][g * 4 + 0], acc[tn][tm][g * 4 + 1], acc[tn][tm][g * 4 + 2],
                     acc[tn][tm][g * 4 + 3]};
          *reinterpret_cast<f32x4*>(dst + n) = v;
        }
    } else if (p.epilogue == EPI_SWIGLU) {
#pragma unroll
      for (int tn = 0; tn < TN; tn += 2)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int j = (n0 + wn0 + tn * 32) / 2 + g * 8 + kg * 4;
          if (j < p.N_store) {
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e)
              o[e] = (bf16)(silu_f(acc[tn][tm][g * 4 + e]) * acc[tn + 1][tm][g * 4 + e]);
            *reinterpret_cast<bf16x4*>(p.out + (int64_t)m * p.ldo + j) = o;
          }
        }
    } else {
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int n = n0 + wn0 + tn * 32 + g * 8 + kg * 4;
          if (n < p.N_store) {
            float v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = acc[tn][tm][g * 4 + e];
            if (p.epilogue == EPI_RESIDUAL) {
              bf16x4 r = *reinterpret_cast<const bf16x4*>(p.residual + (int64_t)m * p.ldr + n);
#pragma unroll
              for (int e = 0; e < 4; ++e) v[e] += (float)r[e];
            }
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (bf16)v[e];
            *reinterpret_cast<bf16x4*>(p.out + (int64_t)m * p.ldo + n) = o;
          }
        }
    }
  }
}

// Sum the split-K partials and apply the epilogue.  One thread per 4 output columns.
__global__ __launch_bounds__(256) void gemm_reduce_kernel(const GemmParams p, int out_cols) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int groups = out_cols / 4;
  if (idx >= (int64_t)p.M * groups) return;
  const int m = (int)(idx / groups);
  const int j = (int)(idx % groups) * 4;
  auto sum_at = [&](int n) {
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    for (int z = 0; z < p.splits; ++z)
      s += *reinterpret_cast<const f32x4*>(p.ws + ((int64_t)z * p.M + m) * p.Npad + n);
    return s;
  };
  bf16x4 o;
  if (p.epilogue == EPI_SWIGLU) {
    const int ng = (j / 32) * 64 + (j % 32);
    f32x4 g = sum_at(ng), u = sum_at(ng + 32);
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = (bf16)(silu_f(g[e]) * u[e]);
  } else {
    f32x4 v = sum_at(j);
    if (p.epilogue == EPI_RESIDUAL) {
      bf16x4 r = *reinterpret_cast<const bf16x4*>(p.residual + (int64_t)m * p.ldr + j);
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] += (float)r[e];
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = (bf16)v[e];
  }
  *reinterpret_cast<bf16x4*>(p.out + (int64_t)m * p.ldo + j) = o;
}

struct TileInfo {
  int bm, bn, lds_bytes, wg_per_cu;
};
static const TileInfo kTiles[5] = {
    {0, 0, 0, 0},
    {256, 256, 2 * (256 + 256) * 128, 1},
    {128, 128, 2 * (128 + 128) * 128, 2},
    {64, 128, 2 * (64 + 128) * 128, 3},
    {32, 256, 2 * (32 + 256) * 128, 2},
};

hipError_t gemm_setup() {
  hipError_t e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<256, 256, 2, 2>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, kTiles[1].lds_bytes);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<128, 128, 2, 2>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, kTiles[2].lds_bytes);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<64, 128, 2, 2>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, kTiles[3].lds_bytes);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<32, 256, 1, 4>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, kTiles[4].lds_bytes);
  return e;
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s) {
  if (a.M <= 0) return hipSuccess;
  int t = a.force_tile;
  if (t < 1 || t > 4) t = a.M <= 32 ? 4 : a.M <= 64 ? 3 : a.M <= 128 ? 2 : 1;
  const TileInfo& ti = kTiles[t];
  GemmParams p;
  p.A = (const bf16*)a.A;
  p.W = (const bf16*)a.W;
  p.out = (bf16*)a.out;
  p.residual = (const bf16*)a.residual;
  p.ws = a.workspace;
  p.lda = a.lda;
  p.Kpad = a.Kpad;
  p.Npad = a.Npad;
  p.ldo = a.ldo;
  p.ldr = a.ldr;
  p.M = a.M;
  p.N_store = a.N_store;
  p.epilogue = a.epilogue;
  p.k_tiles_total = (int)(a.Kpad / 64);
  p.tiles_m = (a.M + ti.bm - 1) / ti.bm;
  p.tiles_n = (int)(a.Npad / ti.bn);
  const int tiles = p.tiles_m * p.tiles_n;
  int splits = a.force_splits;
  if (splits <= 0) {
    splits = 1;
    if (a.M <= 512) {
      const int target = 256 * ti.wg_per_cu;
      splits = target / tiles;
      if (splits > p.k_tiles_total / 4) splits = p.k_tiles_total / 4;
      if (splits < 1) splits = 1;
    }
  }
  if (splits > p.k_tiles_total) splits = p.k_tiles_total;
  while (splits > 1 && (int64_t)splits * a.M * a.Npad > a.workspace_elems) --splits;
  p.k_tiles_per_split = (p.k_tiles_total + splits - 1) / splits;
  splits = (p.k_tiles_total + p.k_tiles_per_split - 1) / p.k_tiles_per_split;
  p.splits = splits;

  dim3 grid(tiles, splits), block(256);
  switch (t) {
    case 1: gemm_kernel<256, 256, 2, 2><<<grid, block, ti.lds_bytes, s>>>(p); break;
    case 2: gemm_kernel<128, 128, 2, 2><<<grid, block, ti.lds_bytes, s>>>(p); break;
    case 3: gemm_kernel<64, 128, 2, 2><<<grid, block, ti.lds_bytes, s>>>(p); break;
    default: gemm_kernel<32, 256, 1, 4><<<grid, block, ti.lds_bytes, s>>>(p); break;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (splits > 1) {
    const int out_cols = a.epilogue == EPI_SWIGLU ? (int)(a.Npad / 2) : a.N_store;
    const int64_t n_thr = (int64_t)a.M * (out_cols / 4);
    gemm_reduce_kernel<<<(unsigned)((n_thr + 255) / 256), 256, 0, s>>>(p, out_cols);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace tdp
