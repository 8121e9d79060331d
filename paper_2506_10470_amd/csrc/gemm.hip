// bf16 MFMA GEMM for the stage's four projections (paper Sec. 3.4: linear layers dominate the
// execution time of a decode step, and only the batch size sets their cost).
//
//   out[M, N] = epilogue( A[M, K] * W^T ),   A bf16 M x K,  W bf16 Npad x Kpad  (both K-contiguous in
//   32-column blocks; W and the stage's own activations are pair-interleaved, see OperandLayout)
//
// Both operands are K-contiguous, so an MFMA fragment is one 16-byte load.  The product is formed
// transposed, D[n][m] = sum_k W[n][k] A[m][k], with the weights as the MFMA "A" operand: a lane
// then holds four consecutive output columns n of one row m, which makes the epilogue's stores
// 8 bytes wide and lets the SwiGLU epilogue find gate and up of one column in the same lane.
//
// Tiles go from global memory straight into LDS (direct-to-LDS loads, a ring of 32-wide k-stages,
// one barrier per stage) with an XOR swizzle of the 16-byte chunks applied on the global side, so
// that the fragment reads are free of bank conflicts.  For small M (decode) the K range is split
// across workgroups; the fp32 partials are summed by the kernel that consumes the projection, or
// by a reduce kernel that applies the epilogue.
#include <stdio.h>
#include <stdlib.h>

#include <initializer_list>
#include <mutex>
#include <unordered_map>

#include "tdp_device.h"
#include "tdp_kernels.h"

namespace tdp {

struct GemmParams {
  const bf16* A;
  const bf16* W;
  bf16* out;
  const void* residual;  // bf16, or fp32 when res_f32
  const float* bias;     // fp32 [Npad] or null
  float* ws;
  OperandLayout a_lay, w_lay, u_lay;
  int64_t Kpad, Npad, ldo, ldr;
  int M, N_store, epilogue, out_f32, res_f32;
  int k_tiles_total, k_tiles_per_split, splits;
  int tiles_m, tiles_n;
  int sb_m, sb_n, n_sb_n, n_sb;  // super-blocks of sb_m x sb_n tiles (at most one XCD's worth, 32)
};

// silu(z) = z / (1 + e^-z), with the hardware reciprocal (1 ulp) in place of an IEEE division: the
// gated epilogue evaluates it 128 times per lane and tile, and its result is rounded to bf16 anyway.
__device__ __forceinline__ float silu_f(float z) { return z * __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }

// Residual add and store of four consecutive output columns (plain / residual epilogues).
__device__ __forceinline__ void store_row4(const GemmParams& p, int m, int n, float (&v)[4]) {
  if (p.bias) {
    const f32x4 b = *reinterpret_cast<const f32x4*>(p.bias + n);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] += b[e];
  }
  if (p.epilogue == EPI_RESIDUAL) {
    if (p.res_f32) {
      const f32x4 r = *reinterpret_cast<const f32x4*>((const float*)p.residual + (int64_t)m * p.ldr + n);
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] += r[e];
    } else {
      const bf16x4 r = *reinterpret_cast<const bf16x4*>((const bf16*)p.residual + (int64_t)m * p.ldr + n);
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] += (float)r[e];
    }
  }
  if (p.out_f32) {
    *reinterpret_cast<f32x4*>((float*)p.out + (int64_t)m * p.ldo + n) = f32x4{v[0], v[1], v[2], v[3]};
  } else {
    bf16x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = (bf16)v[e];
    *reinterpret_cast<bf16x4*>(p.out + (int64_t)m * p.ldo + n) = o;
  }
}

// Epilogue of the GEMM kernel (16x16 accumulator tiles): a lane holds, for each (wt, at), output columns
// n..n+3 of row m, with m = row0 + at*16 + l16 and n = col0 + wt*16 + kq*4.  Gate and up rows
// alternate in blocks of 32 weight rows, i.e. tiles wt, wt+1 (gate) pair with wt+2, wt+3 (up).
template <int AT, int WT>
__device__ __forceinline__ void gemm_epilogue16(const GemmParams& p, f32x4 (&acc)[WT][AT], int row0, int col0,
                                                int l16, int kq, int split) {
#pragma unroll
  for (int at = 0; at < AT; ++at) {
    const int m = row0 + at * 16 + l16;
    if (m >= p.M) continue;
    if (p.splits > 1) {
      float* dst = p.ws + ((int64_t)split * p.M + m) * p.Npad;
#pragma unroll
      for (int wt = 0; wt < WT; ++wt) *reinterpret_cast<f32x4*>(dst + col0 + wt * 16 + kq * 4) = acc[wt][at];
    } else if (p.epilogue == EPI_SWIGLU) {
#pragma unroll
      for (int wt = 0; wt < WT; wt += 4)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int j = (col0 + wt * 16) / 2 + h * 16 + kq * 4;
          if (j < p.N_store) {
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (bf16)(silu_f(acc[wt + h][at][e]) * acc[wt + h + 2][at][e]);
            *reinterpret_cast<bf16x4*>(p.out + operand_offset(p.u_lay, m, j)) = o;
          }
        }
    } else {
#pragma unroll
      for (int wt = 0; wt < WT; ++wt) {
        const int n = col0 + wt * 16 + kq * 4;
        if (n < p.N_store) {
          float v[4] = {acc[wt][at][0], acc[wt][at][1], acc[wt][at][2], acc[wt][at][3]};
          store_row4(p, m, n, v);
        }
      }
    }
  }
}

// The residual epilogue of a whole tile (no split-K, no bias): out = acc + residual.  The residual of
// half the wave's tile is requested in one go - addresses clamped into the matrix instead of guarded,
// so that nothing but loads stands between the first request and the last - and only then added and
// stored: fetched row block by row block behind guards, the loads of one row block were all that
// was ever in flight, and the eight round trips took 45 us per 256 x 256 tile against 12 us for the
// epilogue without a residual (measured; the registers that held the operand fragments are free here).
template <int AT, int WT>
__device__ __forceinline__ void gemm_epilogue16_residual(const GemmParams& p, f32x4 (&acc)[WT][AT], int row0,
                                                         int col0, int l16, int kq) {
  constexpr int AB = AT >= 4 ? 4 : AT;  // row blocks per batch
  const int n_last = p.N_store - 4;
#pragma unroll
  for (int a0 = 0; a0 < AT; a0 += AB) {
    f32x4 r[AB][WT];
#pragma unroll
    for (int ab = 0; ab < AB; ++ab) {
      const int m = min(row0 + (a0 + ab) * 16 + l16, p.M - 1);
#pragma unroll
      for (int wt = 0; wt < WT; ++wt) {
        const int n = min(col0 + wt * 16 + kq * 4, n_last);
        if (p.res_f32) {
          r[ab][wt] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>((const float*)p.residual + (int64_t)m * p.ldr + n));
        } else {
          const bf16x4 t = *reinterpret_cast<const bf16x4*>((const bf16*)p.residual + (int64_t)m * p.ldr + n);
          r[ab][wt] = f32x4{(float)t[0], (float)t[1], (float)t[2], (float)t[3]};
        }
      }
    }
#pragma unroll
    for (int ab = 0; ab < AB; ++ab) {
      const int m = row0 + (a0 + ab) * 16 + l16;
#pragma unroll
      for (int wt = 0; wt < WT; ++wt) {
        const int n = col0 + wt * 16 + kq * 4;
        if (m < p.M && n < p.N_store) {
          const f32x4 v = acc[wt][a0 + ab] + r[ab][wt];
          if (p.out_f32) {
            *reinterpret_cast<f32x4*>((float*)p.out + (int64_t)m * p.ldo + n) = v;
          } else {
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (bf16)v[e];
            *reinterpret_cast<bf16x4*>(p.out + (int64_t)m * p.ldo + n) = o;
          }
        }
      }
    }
  }
}

// Workgroup -> (tile_m, tile_n, split).  Workgroups are dealt round-robin to the 8 XCDs, each
// with its own L2, so the workgroups an XCD runs at once are given one compact sb_m x sb_n block
// of tiles: they then share sb_m activation panels and sb_n weight panels in that L2.  Super-blocks
// are numbered split-major, so with split-K an XCD also keeps to one K range.
__device__ __forceinline__ bool gemm_tile_of_block(const GemmParams& p, int& tile_m, int& tile_n, int& split) {
  const int xcd = blockIdx.x & 7;
  const int local = blockIdx.x >> 3;
  const int sb_size = p.sb_m * p.sb_n;
  const int sb_global = (local / sb_size) * 8 + xcd;
  if (sb_global >= p.n_sb * p.splits) return false;
  split = sb_global / p.n_sb;
  const int sb = sb_global % p.n_sb;
  const int within = local % sb_size;
  tile_m = (sb / p.n_sb_n) * p.sb_m + within % p.sb_m;
  tile_n = (sb % p.n_sb_n) * p.sb_n + within / p.sb_m;
  return tile_m < p.tiles_m && tile_n < p.tiles_n;
}

// The same pipeline on v_mfma_f32_16x16x32_bf16: a stage of 32 k is exactly one MFMA k-step, a wave
// tile of (TM*32) x (TN*32) is (TM*2) x (TN*2) accumulators of four registers.  Operand bytes read
// from LDS per flop are the same as with 32x32x16 tiles, but the accumulator traffic in the
// register file is half, and on a power-limited part that buys clock: with random operands an
// MFMA-only loop sustains 2.16 PFLOP/s with 16x16x32 against 1.89 with 32x32x16 (measured).
// Fragments of stage t+1 are read under the MFMAs of stage t (two register sets, the stage loop
// is unrolled by two); one barrier per stage, at its start.
//
// WNT: the weight tiles are requested as non-temporal.  With a single row of tiles (M up to the tile's
// rows: the decode sizes) every weight byte is read by exactly one workgroup, so keeping it in L2
// only evicts what is shared - the activation panel, the split-K partials.  Measured at M = 32 ... 256
// on the 70B shapes: +6 to +12 % on the down projection, +2 to +8 % on gate/up, +1 to +4 % on QKV and
// O.  With more tile rows the weights are shared through L2 and the hint costs 5-10 % on the large
// shapes; the one exception that pays is two tile rows on a wide projection without split-K (gate/up at
// M = 512: the two readers of a weight tile are neighbours in one super-block and run at the same time,
// so the second read still finds the line): -1.8 %.
template <int BM, int NS, int TM, int TN, int BN = 256, bool WNT = false>
__global__ __launch_bounds__((BM / (TM * 32)) * (BN / 32 / TN) * 64) void gemm_mi16_kernel(const GemmParams p) {
  constexpr int BK = 32;
  constexpr int WAVES_N = BN / 32 / TN, WAVES = (BM / (TM * 32)) * WAVES_N;
  constexpr int CPR = BK / 8;         // 16-byte chunks per row
  // Rows that share one swizzle value.  A fragment read of this kernel is 16 rows x 4 chunks (lane =
  // chunk * 16 + row); measured with SQ_LDS_BANK_CONFLICT on that pattern: the chunk position must
  // turn every 2 rows to be conflict free (4 LDS cycles per ds_read_b128); turning every 4 rows -
  // right for the 32 rows x 2 chunks of the 32x32 kernels - costs 8 cycles per read here.
  constexpr int RW = 2;
  constexpr int RPI = 64 / CPR;       // rows per DMA instruction
  constexpr int IPA = (BM / RPI) / WAVES, IPW = (BN / RPI) / WAVES;
  static_assert(IPA >= 1 && (BM / RPI) % WAVES == 0 && (BN / RPI) % WAVES == 0, "row blocks divide among waves");
  constexpr int STAGE = (BM + BN) * BK;
  constexpr int AT = TM * 2, WT = TN * 2;  // 16-row tiles per wave
  static_assert(WT % 4 == 0, "gate/up pairing");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16* smem = reinterpret_cast<bf16*>(smem_raw);  // [NS][BM + BN][BK]

  int tile_m, tile_n, split;
  if (!gemm_tile_of_block(p, tile_m, tile_n, split)) return;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave / WAVES_N) * (TM * 32);
  const int wn0 = (wave % WAVES_N) * (TN * 32);
  const int l16 = lane & 15;
  const int kq = lane >> 4;
  const int m0 = tile_m * BM;
  const int n0 = tile_n * BN;
  const int kt_begin = split * p.k_tiles_per_split * 2;
  int kt_end = kt_begin + p.k_tiles_per_split * 2;
  if (kt_end > p.k_tiles_total * 2) kt_end = p.k_tiles_total * 2;
  const int n_stages = kt_end - kt_begin;  // even: two stages per 64-wide k-tile

  // DMA addressing: a wave-uniform 64-bit base per operand, which moves one k-stage per request,
  // plus loop-invariant 32-bit per-lane byte offsets (scalar base + vector offset needs no vector
  // arithmetic per load).
  typedef const __attribute__((address_space(1))) char* gptr;
  const int r_in = lane / CPR;
  // Instruction j of an operand lands 1 KiB further on in LDS than instruction 0; that distance
  // rides in the instruction's immediate offset, which also moves the global address, so it is
  // taken out of the per-lane offsets again.  The per-lane offset is zero-extended by the hardware
  // and must not go negative: a constant bias keeps it positive and is subtracted from the bases.
  constexpr int kImmBias = 3 * 1024;
  unsigned a_goff[IPA];  // bytes
#pragma unroll
  for (int j = 0; j < IPA; ++j) {
    const int row = (wave * IPA + j) * RPI + r_in;
    const int c_sw = (lane % CPR) ^ ((row / RW) % CPR);
    // rows past M are computed but never stored; they re-read the tile's valid rows in turn (all of
    // them reading the last valid row makes one hot line for every workgroup of the launch)
    int m = row;
    if (m0 + m > p.M - 1) m = row % (p.M - m0);
    a_goff[j] = 2u * (unsigned)(operand_row_offset(p.a_lay, m) + c_sw * 8) + (unsigned)(kImmBias - j * 1024);
  }
  // weight rows need no clamp; the swizzle term (row / RW) % CPR does not depend on the row block j
  // (RPI is a multiple of RW * CPR)
  static_assert(RPI % (RW * CPR) == 0, "the swizzle repeats per row block");
  unsigned w_goff[IPW];
#pragma unroll
  for (int j = 0; j < IPW; ++j) {
    const int row = (wave * IPW + j) * RPI + r_in;
    const int c_sw = (lane % CPR) ^ ((row / RW) % CPR);
    w_goff[j] = 2u * (unsigned)(operand_row_offset(p.w_lay, row) + c_sw * 8) + (unsigned)(kImmBias - j * 1024);
  }
  const int64_t a_step = 2 * p.a_lay.kb, w_step = 2 * p.w_lay.kb;  // bytes per k-stage
  // the stage being requested: global bases, index and ring slot; past the last stage the bases
  // stay put, so the tail re-fetches the last stage (valid memory, never read)
  gptr a_req = (gptr)(p.A + operand_row_offset(p.a_lay, m0) + (int64_t)kt_begin * p.a_lay.kb) - kImmBias;
  gptr w_req = (gptr)(p.W + operand_row_offset(p.w_lay, n0) + (int64_t)kt_begin * p.w_lay.kb) - kImmBias;
  int req_t = 0, req_slot = 0;
  constexpr int N_DMA = IPA + IPW;
  // One DMA instruction: 64 lanes x 16 bytes from (scalar base + per-lane byte offset) into 1 KiB
  // of LDS at lds_addr.  Written as assembly to get the scalar-base form (no vector address
  // arithmetic per load); M0 carries the LDS address, and every DMA of this kernel goes through
  // here, so nothing else depends on M0.
  auto dma_aim = [](unsigned lds_addr) { asm volatile("s_mov_b32 m0, %0\n\ts_nop 0" ::"s"(lds_addr) : "memory"); };
#define TDP_DMA16(lane_off, base, imm) \
  asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" ::"v"(lane_off), "s"(base), "n"(imm) : "memory")
#define TDP_DMA16W(lane_off, base, imm)                                                                              \
  do {                                                                                                               \
    if constexpr (WNT)                                                                                               \
      asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2 nt" ::"v"(lane_off), "s"(base), "n"(imm) : "memory");   \
    else                                                                                                             \
      asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" ::"v"(lane_off), "s"(base), "n"(imm) : "memory");      \
  } while (0)
  const unsigned ring_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem_raw;
  static_assert(IPA <= 4 && IPW <= 4, "immediate offsets up to 3 KiB");
  // instruction j of the requested stage: activations first, then weights; M0 is aimed at the
  // wave's first KiB of each operand once per stage
  auto dma_one = [&](int j) {
    const unsigned ring = ring_base + req_slot * (STAGE * 2);
    if (j == 0) dma_aim(ring + (wave * IPA * RPI * BK) * 2);
    if (j == IPA) dma_aim(ring + (BM * BK + wave * IPW * RPI * BK) * 2);
    switch (j < IPA ? j : j - IPA) {
      case 0: if (j < IPA) TDP_DMA16(a_goff[0], a_req, 0); else TDP_DMA16W(w_goff[0], w_req, 0); break;
      case 1: if (j < IPA) TDP_DMA16(a_goff[1 % IPA], a_req, 1024); else TDP_DMA16W(w_goff[1 % IPW], w_req, 1024); break;
      case 2: if (j < IPA) TDP_DMA16(a_goff[2 % IPA], a_req, 2048); else TDP_DMA16W(w_goff[2 % IPW], w_req, 2048); break;
      default: if (j < IPA) TDP_DMA16(a_goff[3 % IPA], a_req, 3072); else TDP_DMA16W(w_goff[3 % IPW], w_req, 3072); break;
    }
  };
#undef TDP_DMA16
#undef TDP_DMA16W
  auto dma_advance = [&]() {
    ++req_t;
    if (req_t < n_stages) {
      a_req += a_step;
      w_req += w_step;
    }
    req_slot = req_slot + 1 == NS ? 0 : req_slot + 1;
  };
  auto dma_stage = [&]() {
#pragma unroll
    for (int j = 0; j < N_DMA; ++j) dma_one(j);
    dma_advance();
  };

  f32x4 acc[WT][AT];
#pragma unroll
  for (int wt = 0; wt < WT; ++wt)
#pragma unroll
    for (int at = 0; at < AT; ++at) acc[wt][at] = f32x4{0.f, 0.f, 0.f, 0.f};

  // fragment reads: lane (l16, kq) supplies row l16 of a 16-row tile, k = kq*8 .. +8 of the stage
  // Tile wt / at lies 16 rows = 16 * BK elements further on and 16 is a multiple of RW * CPR, so
  // the swizzle term is the lane's alone: one base per operand, the rest are immediate offsets.
  static_assert(16 % (RW * CPR) == 0, "swizzle repeats every 16 rows");
  const int swz = (kq ^ ((l16 / RW) % CPR)) << 3;
  const int w_off = (BM + wn0 + l16) * BK + swz;
  const int a_off = (wm0 + l16) * BK + swz;
  bf16x8 wf[2][WT], af[2][AT];
  constexpr int PENDING = (NS - 2) * N_DMA;
  static_assert(N_DMA <= WT && AT <= WT && AT >= 4, "one weight tile, one DMA and at most one activation tile per MFMA group");
  int rd_slot = 0;  // ring slot of the stage whose fragments are read next
  int w_next = w_off, a_next = a_off;  // this lane's fragments in that slot (element offsets into smem)
  auto read_frags = [&](int set) {
    const bf16* base = smem + rd_slot * STAGE;
#pragma unroll
    for (int wt = 0; wt < WT; ++wt) wf[set][wt] = ld_bf16x8(base + w_off + wt * 16 * BK);
#pragma unroll
    for (int at = 0; at < AT; ++at) af[set][at] = ld_bf16x8(base + a_off + at * 16 * BK);
  };
  // One stage: its fragments are in register set `set`; the next stage was requested NS-2
  // barriers ago.  The MFMAs are inline assembly so that every accumulator stays in place in its
  // AGPRs (left to itself the register allocator shuttles the 64 accumulator tuples through
  // VGPRs); issue order is therefore explicit: eight groups of MFMAs (one weight tile each), with
  // the fragment reads and the DMA of the stages ahead slotted in behind single MFMAs and pinned
  // by scheduling barriers.
  auto stage = [&](int set) {
    // vmcnt: this wave's loads of the next stage have landed; lgkmcnt: its reads of this stage are
    // complete, so after the barrier this stage's buffer may be refilled and the next one read
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(PENDING) : "memory");
#pragma unroll
    for (int g = 0; g < WT; ++g) {
#pragma unroll
      for (int at = 0; at < AT; ++at) {
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[g][at]) : "v"(wf[set][g]), "v"(af[set][at]));
        // everything that is not an MFMA goes behind single MFMAs, a few instructions at a time, so
        // that it issues while the matrix pipe is busy instead of in a gap of the MFMA stream
        if (at == 0) {
          __builtin_amdgcn_sched_barrier(0);
          wf[set ^ 1][g] = ld_bf16x8(smem + w_next + g * 16 * BK);
          __builtin_amdgcn_sched_barrier(0);
        } else if (at == 1 && g < AT) {
          __builtin_amdgcn_sched_barrier(0);
          af[set ^ 1][g] = ld_bf16x8(smem + a_next + g * 16 * BK);
          __builtin_amdgcn_sched_barrier(0);
        } else if (at == 2 && g < N_DMA) {
          __builtin_amdgcn_sched_barrier(0);
          dma_one(g);
          __builtin_amdgcn_sched_barrier(0);
        }
        // the stage's bookkeeping, behind MFMAs of the last group that carry nothing else: the
        // request side moves on one stage, and so do the fragment offsets.  (The empty statements
        // make the new values exist here rather than wherever their next use is.)
        if (g == WT - 1 && at == 3) {
          __builtin_amdgcn_sched_barrier(0);
          ++req_t;
          if (req_t < n_stages) {
            a_req += a_step;
            w_req += w_step;
          }
          asm volatile("" : "+s"(a_req), "+s"(w_req), "+s"(req_t));
          __builtin_amdgcn_sched_barrier(0);
        }
        if (g == WT - 1 && at == (AT > 4 ? 4 : 3)) {
          __builtin_amdgcn_sched_barrier(0);
          req_slot = req_slot + 1 == NS ? 0 : req_slot + 1;
          rd_slot = rd_slot + 1 == NS ? 0 : rd_slot + 1;
          asm volatile("" : "+s"(req_slot), "+s"(rd_slot));
          __builtin_amdgcn_sched_barrier(0);
        }
        if (g == WT - 1 && at == (AT > 5 ? 5 : 3)) {
          __builtin_amdgcn_sched_barrier(0);
          w_next = rd_slot * STAGE + w_off;
          a_next = rd_slot * STAGE + a_off;
          asm volatile("" : "+v"(w_next), "+v"(a_next));
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
  };

  if (n_stages > 0) {
#pragma unroll
    for (int t = 0; t < NS - 1; ++t) dma_stage();
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(PENDING) : "memory");
    read_frags(0);
    rd_slot = 1 % NS;
    w_next = rd_slot * STAGE + w_off;
    a_next = rd_slot * STAGE + a_off;
    dma_stage();
  }
  for (int t = 0; t < n_stages; t += 2) {
    stage(0);
    stage(1);
  }
  // loads still in flight target LDS only; they must land before the workgroup's LDS is released.
  // The nops cover the MFMA -> accumulator-read distance, which the compiler cannot see.
  asm volatile("s_waitcnt vmcnt(0)\n\ts_nop 15\n\ts_nop 15" ::: "memory");
  if (p.splits == 1 && p.epilogue == EPI_RESIDUAL && !p.bias && p.N_store >= 4)
    gemm_epilogue16_residual<AT, WT>(p, acc, m0 + wm0, n0 + wn0, l16, kq);
  else
    gemm_epilogue16<AT, WT>(p, acc, m0 + wm0, n0 + wn0, l16, kq, split);
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
  if (p.epilogue == EPI_SWIGLU) {
    const int ng = (j / 32) * 64 + (j % 32);
    f32x4 g = sum_at(ng), u = sum_at(ng + 32);
    bf16x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = (bf16)(silu_f(g[e]) * u[e]);
    *reinterpret_cast<bf16x4*>(p.out + operand_offset(p.u_lay, m, j)) = o;
  } else {
    const f32x4 t = sum_at(j);
    float v[4] = {t[0], t[1], t[2], t[3]};
    store_row4(p, m, j, v);
  }
}

struct TileInfo {
  int bm, bn, lds_bytes, wg_per_cu;
};
// kernel variants, selectable through GemmArgs::force_tile (1 .. kGemmTileMax)
static const TileInfo kTiles[kGemmTileMax + 1] = {
    {0, 0, 0, 0},
    {256, 256, 4 * 512 * 64, 1},   // 1: 256 x 256 tile, BK 32 x 4 stages, four waves of 128 x 128
    {128, 256, 6 * 384 * 64, 1},   // 2: 128 x 256 tile, BK 32 x 6 stages, four waves of 64 x 128
    {128, 128, 4 * 256 * 64, 2},   // 3: 128 x 128 tile, BK 32 x 4 stages, four waves of 64 x 64, two workgroups per CU
};

static bool g_print_plan = false;  // tuning aid, read from the environment once (gemm_setup)

hipError_t gemm_setup() {
  static std::once_flag once;
  static hipError_t result = hipSuccess;
  std::call_once(once, [] {
    g_print_plan = getenv("TDP_GEMM_PLAN") != nullptr;
    hipError_t e;
    e = hipSuccess;
    const void* kernels[] = {reinterpret_cast<const void*>(&gemm_mi16_kernel<256, 4, 4, 4, 256, false>),
                             reinterpret_cast<const void*>(&gemm_mi16_kernel<256, 4, 4, 4, 256, true>),
                             reinterpret_cast<const void*>(&gemm_mi16_kernel<128, 6, 2, 4, 256, false>),
                             reinterpret_cast<const void*>(&gemm_mi16_kernel<128, 6, 2, 4, 256, true>),
                             reinterpret_cast<const void*>(&gemm_mi16_kernel<128, 4, 2, 2, 128, false>),
                             reinterpret_cast<const void*>(&gemm_mi16_kernel<128, 4, 2, 2, 128, true>)};
    for (int i = 0; i < 6 && e == hipSuccess; ++i)
      e = hipFuncSetAttribute(kernels[i], hipFuncAttributeMaxDynamicSharedMemorySize, kTiles[1 + i / 2].lds_bytes);
    result = e;
  });
  return result;
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s) {
  if (a.M <= 0) return hipSuccess;
  int t = a.force_tile;
  if (t < 1 || t > kGemmTileMax) {
    // up to 256 rows a projection with few weight rows and a short K fills the chip better with
    // 128-row tiles (twice the workgroups, half the split-K factor); measured at M = 256, K = 8192:
    // 59 vs 72 us (N 10240), 50 vs 61 (N 8192); with K = 28672 the 256-row tile stays ahead (141 vs 148)
    const bool narrow = a.Npad <= 16384 && a.Kpad <= 16384;
    t = a.M <= 128 ? 2 : (a.M <= 256 && narrow) ? 2 : 1;
  }
  const TileInfo& ti = kTiles[t];
  GemmParams p;
  p.A = (const bf16*)a.A;
  p.W = (const bf16*)a.W;
  p.out = (bf16*)a.out;
  p.residual = a.residual;
  p.bias = a.epilogue == EPI_SWIGLU ? nullptr : a.bias;
  p.out_f32 = a.epilogue == EPI_SWIGLU ? 0 : a.out_f32;
  p.res_f32 = a.residual_f32;
  p.ws = a.workspace;
  p.a_lay = a.a_layout;
  p.w_lay = layout_weights(a.Kpad);
  p.u_lay = a.u_layout;
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
  // ---- plan: split-K factor and super-block size ---------------------------------------------
  // The model: an XCD (32 CUs) works through the tiles dealt to it, wg_per_cu * 32 at a time, and a
  // tile costs its k-tiles; split-K adds the fp32 partial round trip.  Small problems (decode) want
  // every XCD equally loaded; large ones want 32-tile super-blocks for L2 reuse.
  // The search below costs tens of microseconds on the host and its answer depends only on the
  // problem's shape, so it is remembered (a serving loop asks for the same few shapes every step).
  struct PlanKey {
    int M, t, force_splits;
    int64_t Npad, Kpad, ws_elems;
    bool operator==(const PlanKey& o) const {
      return M == o.M && t == o.t && force_splits == o.force_splits && Npad == o.Npad && Kpad == o.Kpad &&
             ws_elems == o.ws_elems;
    }
  };
  struct PlanKeyHash {
    size_t operator()(const PlanKey& k) const {
      uint64_t h = 0x9e3779b97f4a7c15ull;
      for (uint64_t v : {(uint64_t)k.M, (uint64_t)k.t, (uint64_t)k.force_splits, (uint64_t)k.Npad, (uint64_t)k.Kpad,
                         (uint64_t)k.ws_elems})
        h = (h ^ v) * 0xff51afd7ed558ccdull + (h >> 29);
      return (size_t)h;
    }
  };
  struct PlanEntry {
    int splits, sb;
  };
  static std::mutex plan_mutex;
  static std::unordered_map<PlanKey, PlanEntry, PlanKeyHash> plan_cache;
  const PlanKey key{a.M, t, a.force_splits, a.Npad, a.Kpad, a.workspace_elems};
  int best_splits = 0, best_sb = 1;
  {
    std::lock_guard<std::mutex> lock(plan_mutex);
    const auto it = plan_cache.find(key);
    if (it != plan_cache.end()) {
      best_splits = it->second.splits;
      best_sb = it->second.sb;
    }
  }
  if (best_splits == 0) {
    best_splits = 1;
    int max_splits = 1;
    if (a.force_splits > 0) max_splits = a.force_splits;
    else if (a.M <= 512) max_splits = p.k_tiles_total / 4 < 16 ? (p.k_tiles_total / 4 > 0 ? p.k_tiles_total / 4 : 1) : 16;
    if (max_splits > p.k_tiles_total) max_splits = p.k_tiles_total;
    double best_cost = 1e300;
    for (int sp = a.force_splits > 0 ? max_splits : 1; sp <= max_splits; ++sp) {
      if (sp > 1 && (int64_t)sp * a.M * a.Npad > a.workspace_elems) break;
      const int per = (p.k_tiles_total + sp - 1) / sp;
      const int real_sp = (p.k_tiles_total + per - 1) / per;
      if (real_sp != sp && a.force_splits <= 0) continue;  // same schedule as a smaller factor
      for (int sb_size = 32; sb_size >= 1; sb_size >>= 1) {
        int sb_m = p.tiles_m >= 4 ? 4 : p.tiles_m >= 2 ? 2 : 1;
        if (sb_m > sb_size) sb_m = sb_size;
        const int sb_n = sb_size / sb_m;
        const int n_sb_n = (p.tiles_n + sb_n - 1) / sb_n;
        const int n_sb_m = (p.tiles_m + sb_m - 1) / sb_m;
        const int n_sb = n_sb_m * n_sb_n;
        int64_t load[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int g = 0; g < n_sb * real_sp; ++g) {
          const int sb = g % n_sb;
          const int rows = (sb / n_sb_n + 1) * sb_m <= p.tiles_m ? sb_m : p.tiles_m - (sb / n_sb_n) * sb_m;
          const int cols = (sb % n_sb_n + 1) * sb_n <= p.tiles_n ? sb_n : p.tiles_n - (sb % n_sb_n) * sb_n;
          load[g & 7] += (int64_t)rows * cols;
        }
        int64_t mx = 0;
        for (int x = 0; x < 8; ++x) mx = load[x] > mx ? load[x] : mx;
        const int slots = 32 * ti.wg_per_cu;
        const double rounds = (double)((mx + slots - 1) / slots);
        // a workgroup pays its pipeline fill and its epilogue whatever its share of K: about 6 k-tiles' worth
        // (without this term the model splits a 224-tile launch eight ways to fill 256 CUs: measured 25 % slower)
        double cost = rounds * (per + 6.0);
        // fp32 partials: 8 bytes per element and split at ~4 TB/s, in units of one k-tile round (~1.8 us)
        if (real_sp > 1) cost += 1.1e-6 * real_sp * a.M * (double)a.Npad + 2.0;
        cost *= 1.0 + 0.02 * (5 - __builtin_ctz(sb_size));  // prefer larger super-blocks on ties
        if (cost < best_cost) {
          best_cost = cost;
          best_splits = real_sp;
          best_sb = sb_size;
        }
      }
    }
    std::lock_guard<std::mutex> lock(plan_mutex);
    if (plan_cache.size() < 65536) plan_cache[key] = PlanEntry{best_splits, best_sb};
  }
  int splits = best_splits;
  p.k_tiles_per_split = (p.k_tiles_total + splits - 1) / splits;
  p.splits = splits;
  p.sb_m = p.tiles_m >= 4 ? 4 : p.tiles_m >= 2 ? 2 : 1;
  if (p.sb_m > best_sb) p.sb_m = best_sb;
  p.sb_n = best_sb / p.sb_m;
  p.n_sb_n = (p.tiles_n + p.sb_n - 1) / p.sb_n;
  p.n_sb = ((p.tiles_m + p.sb_m - 1) / p.sb_m) * p.n_sb_n;
  if (g_print_plan)
    fprintf(stderr, "gemm plan: M=%d N=%lld K=%lld tile=%d tiles=%dx%d splits=%d (k-tiles %d each) super-block %dx%d\n",
            a.M, (long long)a.Npad, (long long)a.Kpad, t, p.tiles_m, p.tiles_n, splits, p.k_tiles_per_split, p.sb_m,
            p.sb_n);
  dim3 grid(((p.n_sb * splits + 7) / 8) * 8 * p.sb_m * p.sb_n);
  // a single row of tiles reads every weight byte once: request them as non-temporal (also two rows of a
  // wide projection, see the kernel's comment)
  const bool wnt = p.tiles_m == 1 || (p.tiles_m == 2 && a.Npad >= 32768 && splits == 1);
  switch (t * 2 + (wnt ? 1 : 0)) {
    case 2: gemm_mi16_kernel<256, 4, 4, 4, 256, false><<<grid, dim3(256), ti.lds_bytes, s>>>(p); break;
    case 3: gemm_mi16_kernel<256, 4, 4, 4, 256, true><<<grid, dim3(256), ti.lds_bytes, s>>>(p); break;
    case 4: gemm_mi16_kernel<128, 6, 2, 4, 256, false><<<grid, dim3(256), ti.lds_bytes, s>>>(p); break;
    case 5: gemm_mi16_kernel<128, 6, 2, 4, 256, true><<<grid, dim3(256), ti.lds_bytes, s>>>(p); break;
    case 6: gemm_mi16_kernel<128, 4, 2, 2, 128, false><<<grid, dim3(256), ti.lds_bytes, s>>>(p); break;
    default: gemm_mi16_kernel<128, 4, 2, 2, 128, true><<<grid, dim3(256), ti.lds_bytes, s>>>(p); break;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const bool defer = a.splits_used != nullptr && a.epilogue != EPI_SWIGLU;
  if (a.splits_used) *a.splits_used = defer ? splits : 1;
  if (splits > 1 && !defer) {
    const int out_cols = a.N_store;  // (gated epilogue: columns of the result, half the weight rows)
    const int64_t n_thr = (int64_t)a.M * (out_cols / 4);
    gemm_reduce_kernel<<<(unsigned)((n_thr + 255) / 256), 256, 0, s>>>(p, out_cols);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace tdp
