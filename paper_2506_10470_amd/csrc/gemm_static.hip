// tdp_gemm_bf16_static: the one-projection diagnostic (tdp_gemm_bf16) for callers that cannot
// allocate device memory - code under HIP graph capture, tight serving loops, harnesses that forbid
// hipMalloc.  The two buffers tdp_gemm_bf16 allocates on every call (the repacked weights and the
// split-K partials) live here in one file-scope device array; the kernels are the same.
//
// `scratch` below is a host-side handle only: its device address is looked up once per device with
// hipGetSymbolAddress and that pointer is what kernels and fills are given.  Every GPU the library
// runs on holds its own copy of the array until the process ends.
#include <stdio.h>
#include <string.h>

#include <mutex>

#include "../../include/tdp.h"
#include "tdp_kernels.h"

namespace tdp {
int probe_fail(int code, const char* msg);  // sets the thread's error message (stage.hip)
}

using namespace tdp;

constexpr int64_t kStaticWeightBytes = 16ll << 20;   // repacked weights: Npad * K bf16 elements
constexpr int64_t kStaticPartialBytes = 48ll << 20;  // split-K partials, fp32
static __device__ __align__(256) unsigned char scratch[kStaticWeightBytes + kStaticPartialBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices];  // per device; null until the first call on that device

int fail_hip(hipError_t e, const char* what) {
  char buf[256];
  snprintf(buf, sizeof buf, "%s: %s", what, hipGetErrorString(e));
  return probe_fail(e == hipErrorOutOfMemory ? TDP_ENOMEM : TDP_EHIP, buf);
}

// The array keeps the last call's contents; what must start at zero is cleared by this kernel (a fill
// kernel rather than a memset, so that the call can also be recorded into a graph).
__global__ __launch_bounds__(256) void fill_zero_kernel(uint4* __restrict__ p, int64_t n16) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n16) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

// device address of this GPU's copy of `scratch` (looked up once per device, with that device current)
int static_scratch(unsigned char** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return probe_fail(TDP_EINVAL, "device ordinal beyond the static scratch table");
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return fail_hip(e, "hipGetSymbolAddress(scratch)");
    if (!p) return probe_fail(TDP_EHIP, "hipGetSymbolAddress returned a null address for the static scratch");
    g_scratch_ptr[dev] = (unsigned char*)p;
  }
  *out = g_scratch_ptr[dev];
  return TDP_OK;
}

int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }

}  // namespace

extern "C" int tdp_gemm_bf16_static(const void* A, const void* W, const void* residual, void* out, int32_t M,
                                    int32_t N, int32_t K, int32_t epilogue, int32_t tile, int32_t splits,
                                    void* stream) {
  if (M < 0 || N <= 0 || K <= 0) return probe_fail(TDP_EINVAL, "bad GEMM shape");
  if (K % 64 || N % 4) return probe_fail(TDP_EINVAL, "K must be a multiple of 64 and N of 4");
  if (epilogue != 0 && epilogue != 1) return probe_fail(TDP_EINVAL, "epilogue must be 0 or 1");
  if (tile < 0 || tile > kGemmTileMax || splits < 0) return probe_fail(TDP_EINVAL, "bad tile / splits");
  const int64_t Npad = round_up(N, 256);
  // the workspace size tdp_gemm_bf16 would allocate, so that both calls plan the launch alike
  const int64_t ws_elems = (int64_t)(splits > 0 ? splits : 16) * M * Npad;
  char buf[200];
  if (Npad * (int64_t)K * 2 > kStaticWeightBytes) {
    snprintf(buf, sizeof buf, "weights of %lld (N rounded up to 256) x %d elements exceed the static scratch (%lld at most)",
             (long long)Npad, (int)K, (long long)(kStaticWeightBytes / 2));
    return probe_fail(TDP_EINVAL, buf);
  }
  if (ws_elems * 4 > kStaticPartialBytes) {
    snprintf(buf, sizeof buf, "split-K workspace of %lld floats exceeds the static scratch (%lld at most)",
             (long long)ws_elems, (long long)(kStaticPartialBytes / 4));
    return probe_fail(TDP_EINVAL, buf);
  }
  if (M == 0) return TDP_OK;
  if (!A || !W || !out || (epilogue == 1 && !residual)) return probe_fail(TDP_EINVAL, "null pointer");
  hipStream_t s = (hipStream_t)stream;
  unsigned char* base = nullptr;
  const int rc = static_scratch(&base);
  if (rc != TDP_OK) return rc;
  hipError_t e = gemm_setup();
  if (e != hipSuccess) return fail_hip(e, "gemm_setup");
  uint16_t* wt = (uint16_t*)base;
  float* ws = (float*)(base + kStaticWeightBytes);
  // weight rows from N up to Npad are computed (never stored): they must read as zeros, as in a fresh buffer
  const int64_t n16 = Npad * (int64_t)K * 2 / 16;
  fill_zero_kernel<<<(unsigned)((n16 + 255) / 256), 256, 0, s>>>((uint4*)wt, n16);
  e = hipGetLastError();
  if (e == hipSuccess) e = launch_repack(W, 0, K, N, wt, K, 0, 0, s);
  if (e == hipSuccess) {
    GemmArgs g;
    memset(&g, 0, sizeof(g));
    g.A = A; g.a_layout = layout_row_major(K); g.W = wt; g.Kpad = K; g.Npad = Npad; g.M = M; g.N_store = N;
    g.out = out; g.ldo = N; g.residual = residual; g.ldr = N;
    g.epilogue = epilogue ? EPI_RESIDUAL : EPI_STORE;
    g.workspace = ws; g.workspace_elems = ws_elems; g.force_tile = tile; g.force_splits = splits;
    e = launch_gemm(g, s);
  }
  if (e != hipSuccess) return fail_hip(e, "tdp_gemm_bf16_static");
  return TDP_OK;
}
