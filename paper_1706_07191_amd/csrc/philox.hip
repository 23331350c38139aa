// Gaussian test matrices drawn on the device (Alg. 2 generates Omega_j on the GPU while the block is
// being transferred, Sec. 3 "Sampling and power iteration").  Counter-based, so any window of rows of
// Omega(seed) can be produced independently and the matrix does not depend on the block partition:
// Philox4x32 with 10 rounds (Salmon et al., SC'11) followed by Box-Muller.
//   element e = row * l + col of the m x l matrix uses output (e & 3) of counter (e >> 2), key = seed;
//   u(x) = ((x >> 9) + 0.5) * 2^-23 (exact in fp32; the transform runs in the output's precision); z0 = sqrt(-2 ln u(x0)) cos(2 pi u(x1)),
//   z1 = the same radius times sin; z2, z3 from (x2, x3).
#include "common.h"

namespace brsvd {

__device__ __forceinline__ void philox_round(uint32_t (&c)[4], uint32_t k0, uint32_t k1) {
  const uint64_t p0 = (uint64_t)0xD2511F53u * c[0];
  const uint64_t p1 = (uint64_t)0xCD9E8D57u * c[2];
  const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c[1] ^ k0;
  const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c[3] ^ k1;
  c[1] = (uint32_t)p1;
  c[3] = (uint32_t)p0;
  c[0] = n0;
  c[2] = n2;
}

template <typename T>
__device__ __forceinline__ T uniform23(uint32_t x) { return ((T)(x >> 9) + T(0.5)) * T(0x1p-23); }

// One thread per counter: four consecutive elements of the dense m x l matrix, scattered into the
// rows [row0, row0 + rows) of a panel with leading dimension ld.
template <typename T>
__global__ void __launch_bounds__(256)
k_philox_normal(T* __restrict__ out, int64_t row0, int64_t rows, int l, int ld, uint32_t key0, uint32_t key1) {
  const int64_t e_beg = row0 * l, e_end = (row0 + rows) * l;
  const int64_t ctr = (e_beg >> 2) + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (ctr * 4 >= e_end) return;
  uint32_t c[4] = {(uint32_t)ctr, (uint32_t)((uint64_t)ctr >> 32), 0u, 0u};
  uint32_t k0 = key0, k1 = key1;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    philox_round(c, k0, k1);
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  T z[4];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    T rad, sn, cs;
    if constexpr (sizeof(T) == 8) {
      rad = sqrt(-2.0 * log(uniform23<double>(c[2 * h])));
      sincospi(2.0 * uniform23<double>(c[2 * h + 1]), &sn, &cs);
    } else {
      rad = sqrtf(-2.0f * logf(uniform23<float>(c[2 * h])));
      sincospif(2.0f * uniform23<float>(c[2 * h + 1]), &sn, &cs);
    }
    z[2 * h] = rad * cs;
    z[2 * h + 1] = rad * sn;
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int64_t e = ctr * 4 + j;
    if (e >= e_beg && e < e_end) {
      const int64_t row = e / l;
      out[(row - row0) * ld + (e - row * l)] = z[j];
    }
  }
}

template <typename T>
__global__ void k_zero_pad_columns(T* __restrict__ out, int64_t rows, int l, int ld) {
  const int pad = ld - l;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= rows * pad) return;
  const int64_t row = idx / pad;
  out[row * ld + l + (idx - row * pad)] = T(0);
}

template <typename T>
int philox_normal(uint64_t seed, int64_t row0, int64_t rows, int l, T* out, int ld, hipStream_t stream) {
  if (rows <= 0 || l <= 0 || ld < l || row0 < 0) return BRSVD_ERR_ARG;
  const int64_t e_beg = row0 * l, e_end = (row0 + rows) * l;
  const int64_t counters = ((e_end + 3) >> 2) - (e_beg >> 2);
  hipLaunchKernelGGL(k_philox_normal<T>, dim3((unsigned)ceil_div(counters, 256)), dim3(256), 0, stream, out, row0, rows,
                     l, ld, (uint32_t)seed, (uint32_t)(seed >> 32));
  if (ld > l)
    hipLaunchKernelGGL(k_zero_pad_columns<T>, dim3((unsigned)ceil_div(rows * (ld - l), 256)), dim3(256), 0, stream, out,
                       rows, l, ld);
  BRSVD_HIP_TRY(hipGetLastError());
  return BRSVD_OK;
}

template int philox_normal<float>(uint64_t, int64_t, int64_t, int, float*, int, hipStream_t);
template int philox_normal<double>(uint64_t, int64_t, int64_t, int, double*, int, hipStream_t);

}  // namespace brsvd
