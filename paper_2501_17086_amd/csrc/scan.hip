// Step (ii) of an iteration: the reverse linear recurrence along the residual
// path, g_l = (e_l + v_l) + lambda_l (.) g_{l+1}, with an fp32 carry.  The
// RMS-norm backward of the block input gradient is fused in front of it
// (v_l = (dn_l - y_l * mean(dn_l (.) y_l)) * rinv_l), so dn is read once and v
// never goes to memory.  HBM-bound: every element is read once and written once.
#include "hbp_common.h"

namespace hbp {

namespace {

// One thread owns 8 consecutive channels of one token and walks down the
// layers; the loads of the next layers do not depend on the carry, so the
// unrolled loop keeps several of them in flight.
template <typename T>
__global__ __launch_bounds__(256) void scan_vec_kernel(ScanArgs a) {
  const long vec_per_layer = a.N * a.d / 8;
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= vec_per_layer) return;
  const long layer = a.N * a.d;
  const long off = idx * 8;
  const long c0 = off % a.d;
  T* g = reinterpret_cast<T*>(a.g);
  const T* dn = reinterpret_cast<const T*>(a.dn);
  const T* e = reinterpret_cast<const T*>(a.e);

  float carry[8];
  load8(g + a.l_hi * layer + off, carry);
#pragma unroll 4
  for (long l = a.l_hi - 1; l >= a.l_lo; --l) {
    float v[8];
    if (dn) {
      load8(dn + l * layer + off, v);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = 0.f;
    }
    if (e) {
      float t[8];
      load8(e + l * layer + off, t);
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] += t[i];
    }
    if (a.lambda) {
      float lam[8];
      load8(a.lambda + l * a.d + c0, lam);
#pragma unroll
      for (int i = 0; i < 8; ++i) carry[i] = fmaf(lam[i], carry[i], v[i]);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) carry[i] += v[i];
    }
    store8(g + l * layer + off, carry);
  }
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// One wavefront owns one token row (all d channels: NCH chunks of 512, 8 per
// lane) so the row reduction of the norm's backward is a wave reduction.
template <typename T, int NCH>
__global__ __launch_bounds__(256) void scan_rows_kernel(ScanArgs a) {
  const int lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (row >= a.N) return;
  const long layer = a.N * a.d;
  T* g = reinterpret_cast<T*>(a.g);
  const T* dn = reinterpret_cast<const T*>(a.dn);
  const T* y = reinterpret_cast<const T*>(a.y);
  const T* e = reinterpret_cast<const T*>(a.e);
  const float inv_d = 1.0f / (float)a.d;

  long off[NCH];
  bool on[NCH];
  float carry[NCH][8];
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    long c = (long)j * 512 + lane * 8;
    on[j] = c < a.d;
    off[j] = row * a.d + c;
    if (on[j]) {
      load8(g + a.l_hi * layer + off[j], carry[j]);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) carry[j][i] = 0.f;
    }
  }

#pragma unroll 2
  for (long l = a.l_hi - 1; l >= a.l_lo; --l) {
    float v[NCH][8], yy[NCH][8];
    float dot = 0.f;
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      if (on[j]) {
        load8(dn + l * layer + off[j], v[j]);
        load8(y + l * layer + off[j], yy[j]);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) { v[j][i] = 0.f; yy[j][i] = 0.f; }
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) dot = fmaf(v[j][i], yy[j][i], dot);
    }
    const float r = a.rinv[l * a.N + row];
    const float m = wave_sum(dot) * inv_d;
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      if (!on[j]) continue;
      float t[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) t[i] = (v[j][i] - yy[j][i] * m) * r;
      if (e) {
        float ee[8];
        load8(e + l * layer + off[j], ee);
#pragma unroll
        for (int i = 0; i < 8; ++i) t[i] += ee[i];
      }
      if (a.lambda) {
        float lam[8];
        load8(a.lambda + l * a.d + (long)j * 512 + lane * 8, lam);
#pragma unroll
        for (int i = 0; i < 8; ++i) carry[j][i] = fmaf(lam[i], carry[j][i], t[i]);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) carry[j][i] += t[i];
      }
      store8(g + l * layer + off[j], carry[j]);
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_fwd_kernel(const T* __restrict__ x, T* __restrict__ y,
                                                          float* __restrict__ rinv, long rows, long d, float eps) {
  const int lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (row >= rows) return;
  const T* xr = x + row * d;
  float ss = 0.f;
  for (long c = lane * 8; c < d; c += 512) {
    float v[8];
    load8(xr + c, v);
#pragma unroll
    for (int i = 0; i < 8; ++i) ss = fmaf(v[i], v[i], ss);
  }
  ss = wave_sum(ss);
  const float r = 1.0f / sqrtf(ss / (float)d + eps);
  if (lane == 0) rinv[row] = r;
  for (long c = lane * 8; c < d; c += 512) {
    float v[8];
    load8(xr + c, v);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] *= r;
    store8(y + row * d + c, v);
  }
}

template <typename T>
hipError_t launch_scan_t(const ScanArgs& a, hipStream_t s) {
  if (a.l_hi <= a.l_lo) return hipSuccess;
  if (a.norm_rms && a.dn) {
    const int nch = (int)((a.d + 511) / 512);
    dim3 grid((unsigned)((a.N + 3) / 4)), block(256);
    switch (nch) {
      case 1: hipLaunchKernelGGL((scan_rows_kernel<T, 1>), grid, block, 0, s, a); break;
      case 2: hipLaunchKernelGGL((scan_rows_kernel<T, 2>), grid, block, 0, s, a); break;
      case 3: hipLaunchKernelGGL((scan_rows_kernel<T, 3>), grid, block, 0, s, a); break;
      case 4: hipLaunchKernelGGL((scan_rows_kernel<T, 4>), grid, block, 0, s, a); break;
      case 5: case 6: hipLaunchKernelGGL((scan_rows_kernel<T, 6>), grid, block, 0, s, a); break;
      case 7: case 8: hipLaunchKernelGGL((scan_rows_kernel<T, 8>), grid, block, 0, s, a); break;
      default: return hipErrorInvalidValue;
    }
  } else {
    const long vecs = a.N * a.d / 8;
    hipLaunchKernelGGL(scan_vec_kernel<T>, dim3((unsigned)((vecs + 255) / 256)), dim3(256), 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_scan(int dtype, const ScanArgs& a, hipStream_t s) {
  return dtype == 0 ? launch_scan_t<float>(a, s) : launch_scan_t<bf16_t>(a, s);
}

hipError_t launch_rmsnorm_fwd(int dtype, const void* x, void* y, float* rinv, long rows, long d, float eps,
                              hipStream_t s) {
  dim3 grid((unsigned)((rows + 3) / 4)), block(256);
  if (dtype == 0)
    hipLaunchKernelGGL(rmsnorm_fwd_kernel<float>, grid, block, 0, s, (const float*)x, (float*)y, rinv, rows, d, eps);
  else
    hipLaunchKernelGGL(rmsnorm_fwd_kernel<bf16_t>, grid, block, 0, s, (const bf16_t*)x, (bf16_t*)y, rinv, rows, d,
                       eps);
  return hipGetLastError();
}

}  // namespace hbp
