// Empirical ceilings of the machine the library runs on, measured with its own trivial kernels:
// how fast HBM can be read (in order, and in the 4 KiB pieces a paged KV cache is read in) and how
// fast the matrix cores run a bf16 MFMA loop with no memory traffic at all.  The benchmark prints
// them next to the published peaks so that a kernel's distance to what the part sustains is on
// record, not only its distance to the datasheet.  Diagnostics: not on the path of any stage call.
#include <stdio.h>

#include <string>

#include "../../include/tdp.h"
#include "tdp_device.h"

namespace tdp {
int probe_fail(int code, const char* msg);  // sets the thread's error message (stage.hip)
}

namespace {

using namespace tdp;

constexpr int kPieceBytes = 4096;    // one (page, kv head) tile of a head_dim-128 bf16 cache
constexpr int kPiecesPerBlock = 4;   // pieces a wave has in flight: 16 KiB, as the decode-attention kernel
constexpr int kBlocksPerWave = 8;

// bijection on [0, 2^bits): odd multiplier, xor-shift, odd multiplier
__device__ __forceinline__ uint32_t scatter_index(uint32_t g, int bits) {
  const uint32_t mask = bits >= 32 ? 0xffffffffu : ((1u << bits) - 1u);
  uint32_t x = (g * 0x9E3779B1u) & mask;
  x ^= x >> ((bits + 1) / 2);
  return (x * 0x85EBCA6Bu) & mask;
}

// Every piece of the first 2^bits * 4 KiB of buf is read exactly once per launch, 16 bytes per lane
// per instruction, sixteen instructions in flight per wave.  scattered = 0: pieces in address order.
// NT: the loads are marked non-temporal (data read once: they need not displace anything in the caches).
template <bool NT>
__global__ __launch_bounds__(256) void hbm_read_probe_kernel(const uint8_t* __restrict__ buf, int bits, int scattered,
                                                             float* __restrict__ sink) {
  const uint32_t wave = (blockIdx.x * 256u + threadIdx.x) >> 6;
  const int lane = threadIdx.x & 63;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
  for (int b = 0; b < kBlocksPerWave; ++b) {
    f32x4 r[kPiecesPerBlock * 4];
#pragma unroll
    for (int j = 0; j < kPiecesPerBlock; ++j) {
      const uint32_t g = (wave * kBlocksPerWave + b) * kPiecesPerBlock + j;
      const uint64_t piece = scattered ? scatter_index(g, bits) : g;
      const uint8_t* p = buf + piece * kPieceBytes + lane * 16;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const f32x4* src = reinterpret_cast<const f32x4*>(p + i * 1024);
        r[j * 4 + i] = NT ? __builtin_nontemporal_load(src) : *src;
      }
    }
#pragma unroll
    for (int j = 0; j < kPiecesPerBlock * 4; ++j) acc += r[j];
  }
  if (acc[0] + acc[1] + acc[2] + acc[3] == 12345.678f) sink[0] = 1.f;  // keeps the loads alive
}

// 16 independent accumulators per wave.  random_operands = 1: operands uniform in (-1, 1) that differ
// from lane to lane and element to element; 0: the same constants everywhere.  The power an MFMA
// draws, and with it the clock the part holds, depends on how many operand bits toggle.
__global__ __launch_bounds__(256) void mfma_probe_kernel(int iters, int random_operands,
                                                         float* __restrict__ sink) {
  const uint32_t t = blockIdx.x * 256u + threadIdx.x;
  bf16x8 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      uint32_t h = (t * 64u + i * 8u + e) * 0x9E3779B1u;
      h ^= h >> 15;
      h *= 0x85EBCA6Bu;
      h ^= h >> 13;
      a[i][e] = random_operands ? (bf16)(((int)(h & 0xffff) - 32768) * (1.0f / 32768.0f)) : (bf16)1.0f;
      b[i][e] = random_operands ? (bf16)(((int)(h >> 16) - 32768) * (1.0f / 32768.0f)) : (bf16)0.0f;
    }
  f32x4 c[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) c[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 16; ++i) c[i] = mfma16(a[i & 3], b[i >> 2], c[i]);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += c[i][0] + c[i][1] + c[i][2] + c[i][3];
  if (s == 12345.678f) sink[0] = 1.f;
}

struct Events {
  hipEvent_t e0 = nullptr, e1 = nullptr;
  ~Events() {
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
  }
};

// ms per launch of `launch`, over `launches` back-to-back launches after one warm-up
template <typename F>
hipError_t time_launches(F launch, int launches, hipStream_t s, float* ms_per_launch) {
  Events ev;
  hipError_t e = hipEventCreate(&ev.e0);
  if (e == hipSuccess) e = hipEventCreate(&ev.e1);
  if (e != hipSuccess) return e;
  launch();
  e = hipEventRecord(ev.e0, s);
  for (int i = 0; i < launches && e == hipSuccess; ++i) {
    launch();
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = hipEventRecord(ev.e1, s);
  if (e == hipSuccess) e = hipEventSynchronize(ev.e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev.e0, ev.e1);
  *ms_per_launch = ms / (float)launches;
  return e;
}

int hip_fail(hipError_t e, const char* what) {
  const std::string msg = std::string(what) + ": " + hipGetErrorString(e);
  return probe_fail(e == hipErrorOutOfMemory ? TDP_ENOMEM : TDP_EHIP, msg.c_str());
}

}  // namespace

extern "C" {

int tdp_probe_hbm_read(const void* buf, int64_t bytes, int32_t pattern, int32_t launches, int64_t* bytes_per_launch,
                       float* ms_per_launch, void* stream) {
  if (!buf || !bytes_per_launch || !ms_per_launch) return probe_fail(TDP_EINVAL, "null pointer");
  if (((uintptr_t)buf & 15) != 0) return probe_fail(TDP_EINVAL, "buf must be 16-byte aligned");
  if (launches < 1 || launches > 1000) return probe_fail(TDP_EINVAL, "launches must be in 1..1000");
  if (pattern < 0 || pattern > 3) return probe_fail(TDP_EINVAL, "pattern must be 0..3 (bit 0: scattered, bit 1: non-temporal)");
  const int scattered = pattern & 1;
  // whole workgroups: 4 waves x 8 blocks x 4 pieces = 128 pieces (512 KiB) each
  constexpr int64_t kMin = 128ll * kPieceBytes;
  if (bytes < kMin) return probe_fail(TDP_EINVAL, "the buffer must hold at least 512 KiB");
  int bits = 7;
  while (bits < 31 && ((int64_t)kPieceBytes << (bits + 1)) <= bytes) ++bits;
  const int64_t pieces = 1ll << bits;
  const unsigned grid = (unsigned)(pieces / 128);
  hipStream_t s = (hipStream_t)stream;
  float* sink = nullptr;
  hipError_t e = hipMalloc((void**)&sink, sizeof(float));
  if (e != hipSuccess) return hip_fail(e, "hipMalloc");
  e = time_launches(
      [&] {
        if (pattern & 2)
          hbm_read_probe_kernel<true><<<grid, 256, 0, s>>>((const uint8_t*)buf, bits, scattered, sink);
        else
          hbm_read_probe_kernel<false><<<grid, 256, 0, s>>>((const uint8_t*)buf, bits, scattered, sink);
      },
      launches, s, ms_per_launch);
  (void)hipFree(sink);
  if (e != hipSuccess) return hip_fail(e, "tdp_probe_hbm_read");
  *bytes_per_launch = pieces * kPieceBytes;
  return TDP_OK;
}

int tdp_probe_mfma_bf16(int32_t iters, int32_t launches, int32_t random_operands, double* flop_per_launch,
                        float* ms_per_launch, void* stream) {
  if (!flop_per_launch || !ms_per_launch) return probe_fail(TDP_EINVAL, "null pointer");
  if (iters < 1 || iters > (1 << 22)) return probe_fail(TDP_EINVAL, "iters must be in 1..2^22");
  if (launches < 1 || launches > 1000) return probe_fail(TDP_EINVAL, "launches must be in 1..1000");
  if (random_operands != 0 && random_operands != 1) return probe_fail(TDP_EINVAL, "random_operands must be 0 or 1");
  hipStream_t s = (hipStream_t)stream;
  int dev = 0, cus = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return hip_fail(e, "device query");
  const unsigned grid = (unsigned)cus * 2;  // two workgroups of four waves per CU: two waves per SIMD
  float* sink = nullptr;
  e = hipMalloc((void**)&sink, sizeof(float));
  if (e != hipSuccess) return hip_fail(e, "hipMalloc");
  e = time_launches([&] { mfma_probe_kernel<<<grid, 256, 0, s>>>(iters, random_operands, sink); }, launches, s, ms_per_launch);
  (void)hipFree(sink);
  if (e != hipSuccess) return hip_fail(e, "tdp_probe_mfma_bf16");
  // per wave and iteration: 16 MFMAs of 16 x 16 x 32 multiply-adds
  *flop_per_launch = (double)grid * 4.0 * (double)iters * 16.0 * (2.0 * 16 * 16 * 32);
  return TDP_OK;
}

}  // extern "C"
