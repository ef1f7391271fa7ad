// Generic strided GEMM with fp32 FMA accumulation: the path for fp32 storage
// and for shapes the MFMA kernels do not cover.  64x64 tile per workgroup,
// 16-deep K slices staged through LDS, 4x4 outputs per thread.
#include "hbp_common.h"

namespace hbp {

namespace {

constexpr int TM = 64, TN = 64, TK = 16, NT = 256;

__device__ __forceinline__ float gelu_f(float a) {
  return 0.5f * a * (1.0f + erff(a * 0.70710678118654752440f));
}
__device__ __forceinline__ float gelu_grad_f(float a) {
  return 0.5f * (1.0f + erff(a * 0.70710678118654752440f)) + a * __expf(-0.5f * a * a) * 0.39894228040143267794f;
}

template <typename T>
__global__ __launch_bounds__(NT) void gemm_generic_kernel(GemmArgs g) {
  __shared__ float As[TK][TM + 4];
  __shared__ float Bs[TK][TN + 4];

  const int tid = threadIdx.x;
  const long bz = blockIdx.z;
  const long batch = bz / g.split_k;
  const int split = (int)(bz % g.split_k);
  const long m0 = (long)blockIdx.y * TM;
  const long n0 = (long)blockIdx.x * TN;

  const T* A = reinterpret_cast<const T*>(g.A) + batch * g.a_sb;
  const T* B = reinterpret_cast<const T*>(g.B) + batch * g.b_sb;

  long kchunk = (g.K + g.split_k - 1) / g.split_k;
  kchunk = (kchunk + TK - 1) / TK * TK;
  const long k_begin = (long)split * kchunk;
  long k_end = k_begin + kchunk;
  if (k_end > g.K) k_end = g.K;

  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  const int tx = tid % 16, ty = tid / 16;
  const bool a_m_fast = (g.a_sm == 1);
  const bool b_n_fast = (g.b_sn == 1);

  for (long k0 = k_begin; k0 < k_end; k0 += TK) {
#pragma unroll
    for (int r = 0; r < (TM * TK) / NT; ++r) {
      int idx = tid + r * NT;
      int mm, kk;
      if (a_m_fast) { mm = idx % TM; kk = idx / TM; } else { kk = idx % TK; mm = idx / TK; }
      long m = m0 + mm, k = k0 + kk;
      float v = 0.f;
      if (m < g.M && k < k_end) v = Elem<T>::load(A + m * g.a_sm + k * g.a_sk);
      As[kk][mm] = v;
    }
#pragma unroll
    for (int r = 0; r < (TN * TK) / NT; ++r) {
      int idx = tid + r * NT;
      int nn, kk;
      if (b_n_fast) { nn = idx % TN; kk = idx / TN; } else { kk = idx % TK; nn = idx / TK; }
      long n = n0 + nn, k = k0 + kk;
      float v = 0.f;
      if (n < g.N && k < k_end) v = Elem<T>::load(B + k * g.b_sk + n * g.b_sn);
      Bs[kk][nn] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }

  // epilogue
  const T* aux = g.aux ? reinterpret_cast<const T*>(g.aux) + batch * g.aux_sb : nullptr;
  T* out2 = g.out2 ? reinterpret_cast<T*>(g.out2) + batch * g.out2_sb : nullptr;
  const float* addf = g.addf ? g.addf + batch * g.addf_sb : nullptr;
  const float* lam = g.lambda ? g.lambda + batch * g.lambda_sb : nullptr;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    long m = m0 + ty * 4 + i;
    if (m >= g.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      long n = n0 + tx * 4 + j;
      if (n >= g.N) continue;
      long off = m * g.ldc + n;
      float v = acc[i][j];
      if (g.split_k > 1) {  // fp32 partial sums [split][batch][M][N]
        float* P = reinterpret_cast<float*>(g.C) + ((long)split * g.batch + batch) * g.c_sb;
        P[off] = v;
        continue;
      }
      if (addf) v += addf[off];
      switch (g.mode) {
        case EPI_MUL_AUX: v *= Elem<T>::load(aux + off); break;
        case EPI_MUL_1MZ2: { float z = Elem<T>::load(aux + off); v *= (1.f - z * z); break; }
        case EPI_ACT_GELU: {
          Elem<T>::store(out2 + off, gelu_grad_f(v));
          v = gelu_f(v);
          break;
        }
        case EPI_ACT_TANH: v = tanhf(v); break;
        case EPI_RESID: {
          float l = lam ? lam[n] : 1.f;
          if (g.lambda_mn) l = Elem<T>::load(reinterpret_cast<const T*>(g.lambda_mn) + batch * g.aux_sb + off);
          v = fmaf(l, Elem<T>::load(aux + off), v);
          break;
        }
        case EPI_ADD_AUX: v += Elem<T>::load(aux + off); break;
        default: break;
      }
      if (g.c_is_f32)
        (reinterpret_cast<float*>(g.C) + batch * g.c_sb)[off] = v;
      else
        Elem<T>::store(reinterpret_cast<T*>(g.C) + batch * g.c_sb + off, v);
    }
  }
}

__global__ void splitk_reduce_kernel(const float* __restrict__ part, float* __restrict__ out, long n, int split) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  long stride = (long)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    float s = 0.f;
    for (int p = 0; p < split; ++p) s += part[(long)p * n + i];
    out[i] = s;
  }
}

}  // namespace

hipError_t launch_gemm_generic(int dtype, const GemmArgs& g, hipStream_t s) {
  dim3 grid((unsigned)((g.N + TN - 1) / TN), (unsigned)((g.M + TM - 1) / TM), (unsigned)(g.batch * g.split_k));
  if (dtype == 0)
    hipLaunchKernelGGL(gemm_generic_kernel<float>, grid, dim3(NT), 0, s, g);
  else
    hipLaunchKernelGGL(gemm_generic_kernel<bf16_t>, grid, dim3(NT), 0, s, g);
  return hipGetLastError();
}

hipError_t launch_splitk_reduce(const float* part, float* out, long n, int split, hipStream_t s) {
  long blocks = (n + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, s, part, out, n, split);
  return hipGetLastError();
}

}  // namespace hbp
