// Elementwise kernels of the recurrent cells whose residual coefficient is a gate.  First the gated recurrent cell (the GRU row of the paper's table of layer
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

// ---------------------------------------------------------------------------
// LSTM (the LSTM row of the same table): state x = [c | h] of width 2H, gates [i | f | o | gg] of width 4H from
// W h + U xin;  c' = f c + i gg,  h' = o tanh(c').  K = diag([f | 0]).
// ---------------------------------------------------------------------------
__device__ __forceinline__ float sigmoidf_(float a) { return 1.f / (1.f + expf(-a)); }

// One step forward: pre [N,4H] fp32; writes gates [N,4H], a [N,2H] = [f | 0], xn [N,2H] = [c' | h'].
template <typename T>
__global__ __launch_bounds__(256) void lstm_fwd_kernel(const float* __restrict__ pre, const T* __restrict__ x,
                                                       T* __restrict__ gates, T* __restrict__ a, T* __restrict__ xn,
                                                       long N, long H) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long per_row = H / 8;
  if (idx >= N * per_row) return;
  const long n = idx / per_row, j = (idx % per_row) * 8;
  float pi[8], pf[8], po[8], pg[8], c[8], i[8], f[8], o[8], gg[8], cn[8], hn[8], zero[8];
  load8(pre + n * 4 * H + j, pi);
  load8(pre + n * 4 * H + H + j, pf);
  load8(pre + n * 4 * H + 2 * H + j, po);
  load8(pre + n * 4 * H + 3 * H + j, pg);
  load8(x + n * 2 * H + j, c);
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    i[q] = sigmoidf_(pi[q]);
    f[q] = sigmoidf_(pf[q]);
    o[q] = sigmoidf_(po[q]);
    gg[q] = tanhf(pg[q]);
    cn[q] = fmaf(f[q], c[q], i[q] * gg[q]);
    hn[q] = o[q] * tanhf(cn[q]);
    zero[q] = 0.f;
  }
  store8(gates + n * 4 * H + j, i);
  store8(gates + n * 4 * H + H + j, f);
  store8(gates + n * 4 * H + 2 * H + j, o);
  store8(gates + n * 4 * H + 3 * H + j, gg);
  store8(a + n * 2 * H + j, f);
  store8(a + n * 2 * H + H + j, zero);
  store8(xn + n * 2 * H + j, cn);
  store8(xn + n * 2 * H + H + j, hn);
}

// Step (i) up to its contraction for `rows` token rows of consecutive blocks.  g = [Gc | Gh] is the gradient of each
// row's NEXT state, x its current state (cell part read), xn its next state (c' read: tanh(c') is recomputed).
//   dct = Gc + Gh o (1 - tanh^2 c')          everything that reaches c'
//   da  = [dct gg i(1-i) | dct c f(1-f) | Gh tanh(c') o(1-o) | dct i (1-gg^2)]
//   vc  = Gh o (1 - tanh^2 c') f (+ e_c)     J's part of d c'/d c (the part that carries Gc is K); cell half of v
template <typename T>
__global__ __launch_bounds__(256) void lstm_vjp_kernel(const T* __restrict__ g, const T* __restrict__ x,
                                                       const T* __restrict__ xn, const T* __restrict__ gates,
                                                       const T* __restrict__ e, T* __restrict__ da,
                                                       T* __restrict__ v, long rows, long H) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long per_row = H / 8;
  if (idx >= rows * per_row) return;
  const long n = idx / per_row, j = (idx % per_row) * 8;
  float Gc[8], Gh[8], c[8], cn[8], i[8], f[8], o[8], gg[8], di[8], df[8], dO[8], dg[8], vc[8];
  load8(g + n * 2 * H + j, Gc);
  load8(g + n * 2 * H + H + j, Gh);
  load8(x + n * 2 * H + j, c);
  load8(xn + n * 2 * H + j, cn);
  load8(gates + n * 4 * H + j, i);
  load8(gates + n * 4 * H + H + j, f);
  load8(gates + n * 4 * H + 2 * H + j, o);
  load8(gates + n * 4 * H + 3 * H + j, gg);
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const float tc = tanhf(cn[q]);
    const float through_h = Gh[q] * o[q] * (1.f - tc * tc);
    const float dct = Gc[q] + through_h;
    di[q] = dct * gg[q] * i[q] * (1.f - i[q]);
    df[q] = dct * c[q] * f[q] * (1.f - f[q]);
    dO[q] = Gh[q] * tc * o[q] * (1.f - o[q]);
    dg[q] = dct * i[q] * (1.f - gg[q] * gg[q]);
    vc[q] = through_h * f[q];
  }
  if (e) {
    float ec[8];
    load8(e + n * 2 * H + j, ec);
#pragma unroll
    for (int q = 0; q < 8; ++q) vc[q] += ec[q];
  }
  store8(da + n * 4 * H + j, di);
  store8(da + n * 4 * H + H + j, df);
  store8(da + n * 4 * H + 2 * H + j, dO);
  store8(da + n * 4 * H + 3 * H + j, dg);
  store8(v + n * 2 * H + j, vc);
}

// ---------------------------------------------------------------------------
// The standard GRU (reset gate included): z = sigmoid(W_z x + U_z xin), r = sigmoid(W_r x + U_r xin),
// n = tanh(W_n (r (.) x) + U_n xin), x' = (1 - z) x + z n.  The candidate's product depends on the reset gate, so a
// step forward is two products with an elementwise kernel after each, and step (i) of the backward pass is
// elementwise -> product with W_n -> elementwise -> product with [W_z; W_r].  Gates are kept as zrn = [z | r | n] [.,3H].
// ---------------------------------------------------------------------------
// forward, first half: pre [N,3H] fp32 (first 2H columns valid): z, r into zrn; rx [N,H] = r (.) x
template <typename T>
__global__ __launch_bounds__(256) void gru_fwd1_kernel(const float* __restrict__ pre, const T* __restrict__ x,
                                                       T* __restrict__ zrn, T* __restrict__ rx, long N, long H) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long per_row = H / 8;
  if (i >= N * per_row) return;
  const long n = i / per_row, j = (i % per_row) * 8;
  float pz[8], pr[8], xv[8], z[8], r[8], o[8];
  load8(pre + n * 3 * H + j, pz);
  load8(pre + n * 3 * H + H + j, pr);
  load8(x + n * H + j, xv);
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    z[q] = sigmoidf_(pz[q]);
    r[q] = sigmoidf_(pr[q]);
    o[q] = r[q] * xv[q];
  }
  store8(zrn + n * 3 * H + j, z);
  store8(zrn + n * 3 * H + H + j, r);
  store8(rx + n * H + j, o);
}
// forward, second half: pre's last H columns = W_n (r (.) x) + U_n xin: n into zrn, a = 1 - z, xn = a x + z n
template <typename T>
__global__ __launch_bounds__(256) void gru_fwd2_kernel(const float* __restrict__ pre, const T* __restrict__ x,
                                                       T* __restrict__ zrn, T* __restrict__ a, T* __restrict__ xn,
                                                       long N, long H) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long per_row = H / 8;
  if (i >= N * per_row) return;
  const long n = i / per_row, j = (i % per_row) * 8;
  float pn[8], xv[8], z[8], nn[8], av[8], o[8];
  load8(pre + n * 3 * H + 2 * H + j, pn);
  load8(x + n * H + j, xv);
  load8(zrn + n * 3 * H + j, z);
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    nn[q] = tanhf(pn[q]);
    av[q] = 1.f - z[q];
    o[q] = fmaf(av[q], xv[q], z[q] * nn[q]);
  }
  store8(zrn + n * 3 * H + 2 * H + j, nn);
  store8(a + n * H + j, av);
  store8(xn + n * H + j, o);
}
// step (i), first elementwise part, for `rows` token rows: da [rows,3H]: columns 0..H = dL/dz through sigmoid',
// columns 2H..3H = dL/dn through tanh' (columns H..2H are written by the second part)
template <typename T>
__global__ __launch_bounds__(256) void gru_vjp1_kernel(const T* __restrict__ g, const T* __restrict__ x,
                                                       const T* __restrict__ zrn, T* __restrict__ da, long rows, long H) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long per_row = H / 8;
  if (i >= rows * per_row) return;
  const long n = i / per_row, j = (i % per_row) * 8;
  float gv[8], xv[8], z[8], nn[8], dz[8], dn[8];
  load8(g + n * H + j, gv);
  load8(x + n * H + j, xv);
  load8(zrn + n * 3 * H + j, z);
  load8(zrn + n * 3 * H + 2 * H + j, nn);
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    dz[q] = gv[q] * (nn[q] - xv[q]) * z[q] * (1.f - z[q]);
    dn[q] = gv[q] * z[q] * (1.f - nn[q] * nn[q]);
  }
  store8(da + n * 3 * H + j, dz);
  store8(da + n * 3 * H + 2 * H + j, dn);
}
// step (i), second elementwise part: drx [rows,H] = dn W_n arrives; da's columns H..2H = drx (.) x (.) r (1 - r);
// drx is overwritten by the state's direct share drx (.) r (+ e); rx (or NULL) = r (.) x for the parameter gradients
template <typename T>
__global__ __launch_bounds__(256) void gru_vjp2_kernel(T* __restrict__ drx, const T* __restrict__ x,
                                                       const T* __restrict__ zrn, const T* __restrict__ e,
                                                       T* __restrict__ da, T* __restrict__ rx, long rows, long H) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long per_row = H / 8;
  if (i >= rows * per_row) return;
  const long n = i / per_row, j = (i % per_row) * 8;
  float dv[8], xv[8], r[8], dr[8], o[8];
  load8(drx + n * H + j, dv);
  load8(x + n * H + j, xv);
  load8(zrn + n * 3 * H + H + j, r);
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    dr[q] = dv[q] * xv[q] * r[q] * (1.f - r[q]);
    o[q] = dv[q] * r[q];
  }
  if (e) {
    float ev[8];
    load8(e + n * H + j, ev);
#pragma unroll
    for (int q = 0; q < 8; ++q) o[q] += ev[q];
  }
  store8(da + n * 3 * H + H + j, dr);
  store8(drx + n * H + j, o);
  if (rx) {
    float rxv[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) rxv[q] = r[q] * xv[q];
    store8(rx + n * H + j, rxv);
  }
}

}  // namespace

hipError_t launch_lstm_fwd(int dtype, const float* pre, const void* x, void* gates, void* a, void* xn, long N, long H,
                           hipStream_t s) {
  const long n = N * (H / 8);
  dim3 grid((unsigned)((n + 255) / 256)), block(256);
  if (dtype == 0)
    hipLaunchKernelGGL(lstm_fwd_kernel<float>, grid, block, 0, s, pre, (const float*)x, (float*)gates, (float*)a,
                       (float*)xn, N, H);
  else
    hipLaunchKernelGGL(lstm_fwd_kernel<bf16_t>, grid, block, 0, s, pre, (const bf16_t*)x, (bf16_t*)gates, (bf16_t*)a,
                       (bf16_t*)xn, N, H);
  return hipGetLastError();
}

hipError_t launch_lstm_vjp(int dtype, const void* g, const void* x, const void* xn, const void* gates, const void* e,
                           void* da, void* v, long rows, long H, hipStream_t s) {
  const long n = rows * (H / 8);
  dim3 grid((unsigned)((n + 255) / 256)), block(256);
  if (dtype == 0)
    hipLaunchKernelGGL(lstm_vjp_kernel<float>, grid, block, 0, s, (const float*)g, (const float*)x, (const float*)xn,
                       (const float*)gates, (const float*)e, (float*)da, (float*)v, rows, H);
  else
    hipLaunchKernelGGL(lstm_vjp_kernel<bf16_t>, grid, block, 0, s, (const bf16_t*)g, (const bf16_t*)x,
                       (const bf16_t*)xn, (const bf16_t*)gates, (const bf16_t*)e, (bf16_t*)da, (bf16_t*)v, rows, H);
  return hipGetLastError();
}

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

#define HBP_GRU_LAUNCH(KERNEL, ROWS, ...)                                                                  \
  do {                                                                                                      \
    const long n_ = (ROWS) * (H / 8);                                                                       \
    dim3 grid((unsigned)((n_ + 255) / 256)), block(256);                                                    \
    hipLaunchKernelGGL(KERNEL<T>, grid, block, 0, s, __VA_ARGS__);                                          \
  } while (0)

hipError_t launch_gru_fwd1(int dtype, const float* pre, const void* x, void* zrn, void* rx, long N, long H, hipStream_t s) {
  if (dtype == 0) { typedef float T; HBP_GRU_LAUNCH(gru_fwd1_kernel, N, pre, (const T*)x, (T*)zrn, (T*)rx, N, H); }
  else { typedef bf16_t T; HBP_GRU_LAUNCH(gru_fwd1_kernel, N, pre, (const T*)x, (T*)zrn, (T*)rx, N, H); }
  return hipGetLastError();
}
hipError_t launch_gru_fwd2(int dtype, const float* pre, const void* x, void* zrn, void* a, void* xn, long N, long H,
                           hipStream_t s) {
  if (dtype == 0) { typedef float T; HBP_GRU_LAUNCH(gru_fwd2_kernel, N, pre, (const T*)x, (T*)zrn, (T*)a, (T*)xn, N, H); }
  else { typedef bf16_t T; HBP_GRU_LAUNCH(gru_fwd2_kernel, N, pre, (const T*)x, (T*)zrn, (T*)a, (T*)xn, N, H); }
  return hipGetLastError();
}
hipError_t launch_gru_vjp1(int dtype, const void* g, const void* x, const void* zrn, void* da, long rows, long H,
                           hipStream_t s) {
  if (dtype == 0) { typedef float T; HBP_GRU_LAUNCH(gru_vjp1_kernel, rows, (const T*)g, (const T*)x, (const T*)zrn, (T*)da, rows, H); }
  else { typedef bf16_t T; HBP_GRU_LAUNCH(gru_vjp1_kernel, rows, (const T*)g, (const T*)x, (const T*)zrn, (T*)da, rows, H); }
  return hipGetLastError();
}
hipError_t launch_gru_vjp2(int dtype, void* drx, const void* x, const void* zrn, const void* e, void* da, void* rx,
                           long rows, long H, hipStream_t s) {
  if (dtype == 0) { typedef float T; HBP_GRU_LAUNCH(gru_vjp2_kernel, rows, (T*)drx, (const T*)x, (const T*)zrn, (const T*)e, (T*)da, (T*)rx, rows, H); }
  else { typedef bf16_t T; HBP_GRU_LAUNCH(gru_vjp2_kernel, rows, (T*)drx, (const T*)x, (const T*)zrn, (const T*)e, (T*)da, (T*)rx, rows, H); }
  return hipGetLastError();
}
#undef HBP_GRU_LAUNCH

}  // namespace hbp
