// The training step around the backward pass: the stand-in loss and its gradient, gradient clipping by global
// norm, and the two optimizers of the paper's training scheme (SGD with momentum and weight decay; AdamW).  All
// elementwise or plain reductions: HBM-bound, a few launches per step.  Reductions are two-stage with fixed
// orders (no atomics): results are bitwise repeatable.
#include "hbp_common.h"

namespace hbp {

namespace {

constexpr int RED_BLOCKS = 1024;   // partial sums per reduction

__device__ __forceinline__ void load4w(const float* p, float (&o)[4]) {
  const float4 t = *reinterpret_cast<const float4*>(p);
  o[0] = t.x; o[1] = t.y; o[2] = t.z; o[3] = t.w;
}
__device__ __forceinline__ void load4w(const bf16_t* p, float (&o)[4]) {
  const uint2 r = *reinterpret_cast<const uint2*>(p);
  o[0] = __uint_as_float(r.x << 16); o[1] = __uint_as_float(r.x & 0xFFFF0000u);
  o[2] = __uint_as_float(r.y << 16); o[3] = __uint_as_float(r.y & 0xFFFF0000u);
}
__device__ __forceinline__ void store4w(float* p, const float (&v)[4]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void store4w(bf16_t* p, const float (&v)[4]) {
  *reinterpret_cast<uint2*>(p) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
}

__device__ __forceinline__ float block_sum(float v, float* sh) {   // 256 threads, fixed tree
  const int tid = threadIdx.x;
  sh[tid] = v;
  __syncthreads();
#pragma unroll
  for (int o = 128; o > 0; o >>= 1) {
    if (tid < o) sh[tid] += sh[tid + o];
    __syncthreads();
  }
  return sh[0];
}

// e = (x - target) / N over `n` elements (8 per thread), partial[b] = this block's sum of (x - target)^2
template <typename T>
__global__ __launch_bounds__(256) void mse_grad_kernel(const T* __restrict__ x, const T* __restrict__ target,
                                                       T* __restrict__ e, long n8, float inv_n, float* __restrict__ partial) {
  __shared__ float sh[256];
  float acc = 0.f;
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n8; i += (long)gridDim.x * 256) {
    float a[8], t[8], o[8];
    load8(x + i * 8, a);
    load8(target + i * 8, t);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float dlt = a[j] - t[j];
      acc = fmaf(dlt, dlt, acc);
      o[j] = dlt * inv_n;
    }
    store8(e + i * 8, o);
  }
  const float s = block_sum(acc, sh);
  if (threadIdx.x == 0) partial[blockIdx.x] = s;
}

template <typename T>
__global__ __launch_bounds__(256) void zero_kernel(T* __restrict__ p, long n8) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= n8) return;
  const float z[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  store8(p + i * 8, z);
}

// partial[b] = sum of g^2 over this block's share (4 per thread and pass)
__global__ __launch_bounds__(256) void sumsq_kernel(const float* __restrict__ g, long n4, float* __restrict__ partial) {
  __shared__ float sh[256];
  float acc = 0.f;
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n4; i += (long)gridDim.x * 256) {
    const float4 v = *reinterpret_cast<const float4*>(g + i * 4);
    acc = fmaf(v.x, v.x, acc); acc = fmaf(v.y, v.y, acc); acc = fmaf(v.z, v.z, acc); acc = fmaf(v.w, v.w, acc);
  }
  const float s = block_sum(acc, sh);
  if (threadIdx.x == 0) partial[blockIdx.x] = s;
}

// out[0] = f(sum of `count` partials), one block, fixed order, double accumulation.
// mode 0: the loss, 0.5 * sum * scale;  mode 1: the clipping factor min(1, max_norm / (sqrt(sum) + 1e-6))
__global__ __launch_bounds__(256) void finalize_kernel(const float* __restrict__ partial, int count, int mode,
                                                       float scale, float* __restrict__ out) {
  __shared__ double sh[256];
  double acc = 0.0;
  for (int i = threadIdx.x; i < count; i += 256) acc += (double)partial[i];
  sh[threadIdx.x] = acc;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double s = sh[0];
    if (mode == 0) out[0] = (float)(0.5 * s * (double)scale);
    else {
      const double f = (double)scale / (sqrt(s) + 1e-6);
      out[0] = (float)(f < 1.0 ? f : 1.0);
    }
  }
}

// One optimizer update of n elements (n % 4 == 0), 4 per thread.  `master` (fp32 copy of the weights) may be NULL:
// the weights are then read from and kept in the storage type alone.  clip: device pointer to the factor on the
// gradient, or NULL for 1.
template <typename T, bool ADAMW>
__global__ __launch_bounds__(256) void optim_kernel(T* __restrict__ w, float* __restrict__ master, const float* __restrict__ g,
                                                    float* __restrict__ m, float* __restrict__ v, long n4,
                                                    const float* __restrict__ clip, OptimArgs o) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= n4) return;
  const float cs = clip ? clip[0] : 1.f;
  float wv[4], gv[4], mv[4], vv[4];
  if (master) {
    const float4 t = *reinterpret_cast<const float4*>(master + i * 4);
    wv[0] = t.x; wv[1] = t.y; wv[2] = t.z; wv[3] = t.w;
  } else {
    load4w(w + i * 4, wv);
  }
  {
    const float4 t = *reinterpret_cast<const float4*>(g + i * 4);
    gv[0] = t.x; gv[1] = t.y; gv[2] = t.z; gv[3] = t.w;
    const float4 u = *reinterpret_cast<const float4*>(m + i * 4);
    mv[0] = u.x; mv[1] = u.y; mv[2] = u.z; mv[3] = u.w;
  }
  if (ADAMW) {
    const float4 u = *reinterpret_cast<const float4*>(v + i * 4);
    vv[0] = u.x; vv[1] = u.y; vv[2] = u.z; vv[3] = u.w;
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (ADAMW) {
      const float gg = cs * gv[j];
      float ww = wv[j] * (1.f - o.lr * o.weight_decay);
      mv[j] = o.beta1 * mv[j] + (1.f - o.beta1) * gg;
      vv[j] = o.beta2 * vv[j] + (1.f - o.beta2) * gg * gg;
      const float mhat = mv[j] * o.inv_bias1, vhat = vv[j] * o.inv_bias2;
      ww -= o.lr * mhat / (sqrtf(vhat) + o.eps);
      wv[j] = ww;
    } else {
      const float gg = cs * gv[j] + o.weight_decay * wv[j];
      mv[j] = o.beta1 * mv[j] + gg;
      wv[j] -= o.lr * mv[j];
    }
  }
  *reinterpret_cast<float4*>(m + i * 4) = make_float4(mv[0], mv[1], mv[2], mv[3]);
  if (ADAMW) *reinterpret_cast<float4*>(v + i * 4) = make_float4(vv[0], vv[1], vv[2], vv[3]);
  if (master) *reinterpret_cast<float4*>(master + i * 4) = make_float4(wv[0], wv[1], wv[2], wv[3]);
  store4w(w + i * 4, wv);
}

}  // namespace

size_t train_scratch_floats() { return 6 * RED_BLOCKS + 16; }

template <typename T>
hipError_t launch_mse_t(const void* x, const void* target, void* e, long n, float inv_n, float* partial, float* loss,
                        hipStream_t s) {
  hipLaunchKernelGGL(mse_grad_kernel<T>, dim3(RED_BLOCKS), dim3(256), 0, s, (const T*)x, (const T*)target, (T*)e, n / 8,
                     inv_n, partial);
  hipLaunchKernelGGL(finalize_kernel, dim3(1), dim3(256), 0, s, partial, RED_BLOCKS, 0, inv_n, loss);
  return hipGetLastError();
}
hipError_t launch_mse_loss_grad(int dtype, const void* x, const void* target, void* e, long n, float inv_n,
                                float* scratch, float* loss, hipStream_t s) {
  return dtype == 0 ? launch_mse_t<float>(x, target, e, n, inv_n, scratch, loss, s)
                    : launch_mse_t<bf16_t>(x, target, e, n, inv_n, scratch, loss, s);
}
hipError_t launch_zero(int dtype, void* p, long n, hipStream_t s) {
  const long n8 = n / 8;
  if (dtype == 0) hipLaunchKernelGGL(zero_kernel<float>, dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, s, (float*)p, n8);
  else hipLaunchKernelGGL(zero_kernel<bf16_t>, dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, s, (bf16_t*)p, n8);
  return hipGetLastError();
}

// factor[0] = min(1, max_norm / (global L2 norm of the given gradients + 1e-6)); up to 5 tensors
hipError_t launch_clip_factor(const float* const* grads, const long* sizes, int count, float max_norm, float* scratch,
                              float* factor, hipStream_t s) {
  for (int t = 0; t < count; ++t)
    hipLaunchKernelGGL(sumsq_kernel, dim3(RED_BLOCKS), dim3(256), 0, s, grads[t], sizes[t] / 4, scratch + (long)t * RED_BLOCKS);
  hipLaunchKernelGGL(finalize_kernel, dim3(1), dim3(256), 0, s, scratch, count * RED_BLOCKS, 1, max_norm, factor);
  return hipGetLastError();
}

hipError_t launch_optim(int dtype, int adamw, void* w, float* master, const float* g, float* m, float* v, long n,
                        const float* clip, const OptimArgs& o, hipStream_t s) {
  const long n4 = n / 4;
  const dim3 grid((unsigned)((n4 + 255) / 256)), block(256);
  if (dtype == 0) {
    if (adamw) hipLaunchKernelGGL((optim_kernel<float, true>), grid, block, 0, s, (float*)w, master, g, m, v, n4, clip, o);
    else hipLaunchKernelGGL((optim_kernel<float, false>), grid, block, 0, s, (float*)w, master, g, m, v, n4, clip, o);
  } else {
    if (adamw) hipLaunchKernelGGL((optim_kernel<bf16_t, true>), grid, block, 0, s, (bf16_t*)w, master, g, m, v, n4, clip, o);
    else hipLaunchKernelGGL((optim_kernel<bf16_t, false>), grid, block, 0, s, (bf16_t*)w, master, g, m, v, n4, clip, o);
  }
  return hipGetLastError();
}

}  // namespace hbp
