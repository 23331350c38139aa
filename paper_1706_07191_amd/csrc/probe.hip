// Measured peaks of the machine the library runs on, for the roofline fractions quoted next to the
// published ones: a streaming read of device memory, and a loop of independent fp32 MFMAs.
// Diagnostic only; nothing on the SVD path calls these.
#include "common.h"

namespace brsvd {

__global__ void __launch_bounds__(256)
k_probe_read(const floatx4* __restrict__ src, int64_t n16, float* __restrict__ sink) {
  floatx4 acc = {0.f, 0.f, 0.f, 0.f};
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) {
    const floatx4 v = __builtin_nontemporal_load(src + i);
    acc += v;
  }
  const float s = acc[0] + acc[1] + acc[2] + acc[3];
  if (s == 12345.678f) sink[0] = s;          // keeps the loads alive; practically never true
}

template <typename T, typename V4>
__device__ __forceinline__ V4 probe_mfma(T a, T b, V4 c);
template <>
__device__ __forceinline__ floatx4 probe_mfma<float, floatx4>(float a, float b, floatx4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// 16 independent accumulators per wave, operands pseudo-random per lane (constant operands draw less
// power and run a few per cent faster).
template <typename T, typename V4>
__global__ void __launch_bounds__(256)
k_probe_mfma(T* __restrict__ out, int iters) {
  V4 acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = V4{T(0), T(0), T(0), T(0)};
  T a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    unsigned h = (blockIdx.x * 256u + threadIdx.x) * 131u + i * 7919u;
    h ^= h >> 16; h *= 0x85ebca6bu; h ^= h >> 13; h *= 0xc2b2ae35u; h ^= h >> 16;
    a[i] = (T)((float)(h & 0xffffff) / 8388608.0f - 1.0f);
    b[i] = (T)((float)((h >> 3) & 0xffffff) / 8388608.0f - 1.0f);
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = probe_mfma<T, V4>(a[i & 7], b[(i * 5 + 1) & 7], acc[i]);
  }
  T s = T(0);
#pragma unroll
  for (int i = 0; i < 16; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

// kind 0: read `amount` bytes (rounded down to 16) from `buf`; kind 1: `amount` fp32 MFMA iterations per
// wave on 2048 workgroups of four waves, writing 2048*256 floats to `buf`.
// *seconds = duration of the one launch (HIP events on `stream`); *work = bytes read or flops done.
int probe(int kind, void* buf, uint64_t amount, double* seconds, double* work, hipStream_t stream) {
  if (!buf || !seconds || !work || amount == 0) return BRSVD_ERR_ARG;
  hipEvent_t e0, e1;
  BRSVD_HIP_TRY(hipEventCreate(&e0));
  BRSVD_HIP_TRY(hipEventCreate(&e1));
  const int grid = 2048;
  int status = BRSVD_OK;
  for (int rep = 0; rep < 2 && status == BRSVD_OK; ++rep) {        // the first launch warms up
    (void)hipEventRecord(e0, stream);
    if (kind == 0) {
      hipLaunchKernelGGL(k_probe_read, dim3(8192), dim3(256), 0, stream, (const floatx4*)buf, (int64_t)(amount / 16),
                         (float*)buf);
      *work = (double)(amount / 16 * 16);
    } else if (kind == 1) {
      hipLaunchKernelGGL((k_probe_mfma<float, floatx4>), dim3(grid), dim3(256), 0, stream, (float*)buf, (int)amount);
      *work = (double)grid * 4 * (double)amount * 16 * 2048.0;
    } else {
      status = BRSVD_ERR_ARG;
      break;
    }
    (void)hipEventRecord(e1, stream);
    if (hipEventSynchronize(e1) != hipSuccess || hipGetLastError() != hipSuccess) { status = BRSVD_ERR_HIP; break; }
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, e0, e1);
    *seconds = ms * 1e-3;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  return status;
}

}  // namespace brsvd
