// Products with very few rows: C[M,N] = epilogue(A[M,K] . B[K,N]) for M of a few dozen, bf16.
//
// Exact backpropagation through time (the sequential baseline of Section 2.1 that Highway-BP is
// compared with) multiplies one time step's [batch, d] gradient by a weight matrix, step after
// step.  A 256 x 256 tile is the wrong tool there: one tile row is mostly padding and the product
// runs on d/256 compute units.  Here a workgroup owns a 32 x 32 block of C, its 4 waves split the
// contraction in quarters, and both operands are read straight from memory into the MFMA operand
// layout (8 consecutive k per lane), which needs both K-contiguous: the weight is passed
// transposed (Bt[n][k]); transpose_bf16 below makes that copy once per backward pass.  The four
// partial blocks are summed through LDS and the epilogue runs on the sum.
#include "hbp_common.h"

namespace hbp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int RED_LD = 36;   // floats per row of a partial block in LDS (16-byte aligned rows, banks spread)

__global__ __launch_bounds__(256) void gemm_skinny_kernel(SkinnyArgs a) {
  __shared__ float red[4][32][RED_LD];
  const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
  const int r = l & 31, h = l >> 5;
  const long n0 = (long)blockIdx.x * 32, m0 = (long)blockIdx.y * 32;
  const long kq = a.K / 4;
  long am = m0 + r;
  if (am > a.M - 1) am = a.M - 1;   // rows past the end repeat the last one; never stored
  const bf16_t* pa = reinterpret_cast<const bf16_t*>(a.A) + am * a.lda + w * kq + 8 * h;
  const bf16_t* pb = reinterpret_cast<const bf16_t*>(a.Bt) + (n0 + r) * a.ldbt + w * kq + 8 * h;
  float16v acc;
#pragma unroll
  for (int q = 0; q < 16; ++q) acc[q] = 0.f;
  const int steps = (int)(kq / 16);
#pragma unroll 8
  for (int s = 0; s < steps; ++s) {
    bf16x8 fa = *reinterpret_cast<const bf16x8*>(pa + 16 * s);
    bf16x8 fb = *reinterpret_cast<const bf16x8*>(pb + 16 * s);
    // operands swapped: the lane owns output row r and, per group of 4 registers, 4 consecutive columns
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb, fa, acc, 0, 0, 0);
  }
#pragma unroll
  for (int qg = 0; qg < 4; ++qg) {
    float4 v = make_float4(acc[4 * qg], acc[4 * qg + 1], acc[4 * qg + 2], acc[4 * qg + 3]);
    *reinterpret_cast<float4*>(&red[w][r][8 * qg + 4 * h]) = v;
  }
  __syncthreads();
  const int row = threadIdx.x >> 3, c0 = (threadIdx.x & 7) * 4;
  if (m0 + row >= a.M) return;
  float v[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    float4 t = *reinterpret_cast<const float4*>(&red[p][row][c0]);
    v[0] += t.x; v[1] += t.y; v[2] += t.z; v[3] += t.w;
  }
  if (a.addf) {
    float4 t = *reinterpret_cast<const float4*>(a.addf + (m0 + row) * a.ldc + n0 + c0);
    v[0] += t.x; v[1] += t.y; v[2] += t.z; v[3] += t.w;
  }
  if (a.mode == EPI_ACT_TANH) {
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = tanhf(v[j]);
  } else if (a.mode != EPI_STORE && a.aux) {
    const bf16_t* px = reinterpret_cast<const bf16_t*>(a.aux) + (m0 + row) * a.ldaux + n0 + c0;
    uint2 raw = *reinterpret_cast<const uint2*>(px);
    float x[4] = {__uint_as_float(raw.x << 16), __uint_as_float(raw.x & 0xFFFF0000u),
                  __uint_as_float(raw.y << 16), __uint_as_float(raw.y & 0xFFFF0000u)};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (a.mode == EPI_MUL_AUX) v[j] *= x[j];
      else if (a.mode == EPI_MUL_1MZ2) v[j] *= (1.f - x[j] * x[j]);
      else v[j] += x[j];
    }
  }
  if (a.mode == EPI_RESID) {   // the residual path's step: + lambda (.) next (with aux = e_l added above when given)
    const long off = (m0 + row) * a.ldc + n0 + c0;
    uint2 raw = *reinterpret_cast<const uint2*>(reinterpret_cast<const bf16_t*>(a.next) + off);
    float x[4] = {__uint_as_float(raw.x << 16), __uint_as_float(raw.x & 0xFFFF0000u),
                  __uint_as_float(raw.y << 16), __uint_as_float(raw.y & 0xFFFF0000u)};
    float lm[4] = {1.f, 1.f, 1.f, 1.f};
    if (a.lambda) {
      float4 t = *reinterpret_cast<const float4*>(a.lambda + n0 + c0);
      lm[0] = t.x; lm[1] = t.y; lm[2] = t.z; lm[3] = t.w;
    } else if (a.lambda_mn) {
      uint2 rl = *reinterpret_cast<const uint2*>(reinterpret_cast<const bf16_t*>(a.lambda_mn) + off);
      lm[0] = __uint_as_float(rl.x << 16); lm[1] = __uint_as_float(rl.x & 0xFFFF0000u);
      lm[2] = __uint_as_float(rl.y << 16); lm[3] = __uint_as_float(rl.y & 0xFFFF0000u);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] += lm[j] * x[j];
  }
  if (a.c_is_f32) {
    *reinterpret_cast<float4*>(reinterpret_cast<float*>(a.C) + (m0 + row) * a.ldc + n0 + c0) =
        make_float4(v[0], v[1], v[2], v[3]);
    return;
  }
  uint2 o;
  o.x = (unsigned)f32_to_bf16(v[0]) | ((unsigned)f32_to_bf16(v[1]) << 16);
  o.y = (unsigned)f32_to_bf16(v[2]) | ((unsigned)f32_to_bf16(v[3]) << 16);
  *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(a.C) + (m0 + row) * a.ldc + n0 + c0) = o;
}

// dst[c][r] = src[r][c], 2-byte elements, 32 x 32 tiles through LDS
__global__ __launch_bounds__(256) void transpose16_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst,
                                                          int rows, int cols) {
  __shared__ bf16_t t[32][34];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int rr = r0 + ty + 8 * i, cc = c0 + tx;
    if (rr < rows && cc < cols) t[ty + 8 * i][tx] = src[(long)rr * cols + cc];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int cc = c0 + ty + 8 * i, rr = r0 + tx;
    if (rr < rows && cc < cols) dst[(long)cc * rows + rr] = t[tx][ty + 8 * i];
  }
}

}  // namespace

bool skinny_ok(long M, long N, long K) {
  return M >= 1 && M <= 128 && N % 32 == 0 && K % 64 == 0 && N >= 32 && K >= 64;
}

hipError_t launch_gemm_skinny(const SkinnyArgs& a, hipStream_t s) {
  if (!skinny_ok(a.M, a.N, a.K)) return hipErrorInvalidValue;
  if (a.mode != EPI_STORE && a.mode != EPI_MUL_AUX && a.mode != EPI_MUL_1MZ2 && a.mode != EPI_ADD_AUX &&
      a.mode != EPI_RESID && a.mode != EPI_ACT_TANH)
    return hipErrorInvalidValue;
  if (a.mode != EPI_STORE && a.mode != EPI_RESID && a.mode != EPI_ACT_TANH && !a.aux) return hipErrorInvalidValue;
  if (a.mode == EPI_RESID && !a.next) return hipErrorInvalidValue;
  if (a.c_is_f32 && a.mode != EPI_STORE) return hipErrorInvalidValue;
  if ((a.lda % 8) || (a.ldbt % 8) || (a.ldc % 4) || (a.aux && (a.ldaux % 4))) return hipErrorInvalidValue;
  dim3 grid((unsigned)(a.N / 32), (unsigned)((a.M + 31) / 32));
  hipLaunchKernelGGL(gemm_skinny_kernel, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_transpose_bf16(const void* src, void* dst, int rows, int cols, hipStream_t s) {
  dim3 grid((unsigned)((cols + 31) / 32), (unsigned)((rows + 31) / 32));
  hipLaunchKernelGGL(transpose16_kernel, grid, dim3(256), 0, s, reinterpret_cast<const bf16_t*>(src),
                     reinterpret_cast<bf16_t*>(dst), rows, cols);
  return hipGetLastError();
}

}  // namespace hbp
