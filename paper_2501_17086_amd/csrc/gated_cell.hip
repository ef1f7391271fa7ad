// Elementwise kernels of the gated recurrent cell (the GRU row of the paper's table of layer
// decompositions: f(x) = a(x) (.) x + b(x), r(x, z) = z1 (.) x + z2) for
//   u = sigmoid(W_u x + U_u xin),  c = tanh(W_c x + U_c xin),  a = 1 - u,  b = u (.) c.
// The two products with the weights are contractions (GEMM kernels); what is left of the cell is
// elementwise and HBM-bound: 8 channels per thread, 16-byte accesses.
#include "hbp_common.h"

namespace hbp {
namespace {

// One step forward.  pre [N,2H] fp32 = [W_u x + U_u xin | W_c x + U_c xin];
// writes uc [N,2H] = [u | c], a [N,H] = 1 - u and xn [N,H] = a (.) x + u (.) c.
template <typename T>
__global__ __launch_bounds__(256) void gated_fwd_kernel(const float* __restrict__ pre, const T* __restrict__ x,
                                                        T* __restrict__ uc, T* __restrict__ a, T* __restrict__ xn,
                                                        long N, long H) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long per_row = H / 8;
  if (i >= N * per_row) return;
  const long n = i / per_row, j = (i % per_row) * 8;
  float pu[8], pc[8], xv[8], u[8], c[8], av[8], o[8];
  load8(pre + n * 2 * H + j, pu);
  load8(pre + n * 2 * H + H + j, pc);
  load8(x + n * H + j, xv);
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    u[q] = 1.f / (1.f + expf(-pu[q]));
    c[q] = tanhf(pc[q]);
    av[q] = 1.f - u[q];
    o[q] = fmaf(av[q], xv[q], u[q] * c[q]);
  }
  store8(uc + n * 2 * H + j, u);
  store8(uc + n * 2 * H + H + j, c);
  store8(a + n * H + j, av);
  store8(xn + n * H + j, o);
}

// Step (i) without its second contraction, for `rows` = blocks x N token rows at once:
// da [rows,2H] = [ g (.) (c - x) (.) u (1 - u) | g (.) u (.) (1 - c^2) ]   (dL/du and dL/dc of r = (1-u) x + u c,
// taken through sigmoid' and tanh'); g is the gradient of the NEXT state of each row.
template <typename T>
__global__ __launch_bounds__(256) void gated_vjp_kernel(const T* __restrict__ g, const T* __restrict__ x,
                                                        const T* __restrict__ uc, T* __restrict__ da, long rows,
                                                        long H) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long per_row = H / 8;
  if (i >= rows * per_row) return;
  const long n = i / per_row, j = (i % per_row) * 8;
  float gv[8], xv[8], u[8], c[8], du[8], dc[8];
  load8(g + n * H + j, gv);
  load8(x + n * H + j, xv);
  load8(uc + n * 2 * H + j, u);
  load8(uc + n * 2 * H + H + j, c);
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    du[q] = gv[q] * (c[q] - xv[q]) * u[q] * (1.f - u[q]);
    dc[q] = gv[q] * u[q] * (1.f - c[q] * c[q]);
  }
  store8(da + n * 2 * H + j, du);
  store8(da + n * 2 * H + H + j, dc);
}

}  // namespace

hipError_t launch_gated_fwd(int dtype, const float* pre, const void* x, void* uc, void* a, void* xn, long N, long H,
                            hipStream_t s) {
  const long n = N * (H / 8);
  dim3 grid((unsigned)((n + 255) / 256)), block(256);
  if (dtype == 0)
    hipLaunchKernelGGL(gated_fwd_kernel<float>, grid, block, 0, s, pre, (const float*)x, (float*)uc, (float*)a,
                       (float*)xn, N, H);
  else
    hipLaunchKernelGGL(gated_fwd_kernel<bf16_t>, grid, block, 0, s, pre, (const bf16_t*)x, (bf16_t*)uc, (bf16_t*)a,
                       (bf16_t*)xn, N, H);
  return hipGetLastError();
}

hipError_t launch_gated_vjp(int dtype, const void* g, const void* x, const void* uc, void* da, long rows, long H,
                            hipStream_t s) {
  const long n = rows * (H / 8);
  dim3 grid((unsigned)((n + 255) / 256)), block(256);
  if (dtype == 0)
    hipLaunchKernelGGL(gated_vjp_kernel<float>, grid, block, 0, s, (const float*)g, (const float*)x, (const float*)uc,
                       (float*)da, rows, H);
  else
    hipLaunchKernelGGL(gated_vjp_kernel<bf16_t>, grid, block, 0, s, (const bf16_t*)g, (const bf16_t*)x,
                       (const bf16_t*)uc, (bf16_t*)da, rows, H);
  return hipGetLastError();
}

}  // namespace hbp
