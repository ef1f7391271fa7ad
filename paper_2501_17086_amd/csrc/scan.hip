// Step (ii) of an iteration: the reverse linear recurrence along the residual
// path, g_l = (e_l + v_l) + lambda_l (.) g_{l+1}, with an fp32 carry.  The
// RMS-norm backward of the block input gradient is fused in front of it
// (v_l = (dn_l - y_l * mean(dn_l (.) y_l)) * rinv_l), so dn is read once and v
// never goes to memory.  HBM-bound: every element is read once and written once.
#include "hbp_common.h"
#include <atomic>
#include <type_traits>

namespace hbp {

namespace {

// One thread owns 8 consecutive channels of one token and walks down the
// layers; the loads of the next layers do not depend on the carry, so the
// unrolled loop keeps several of them in flight.
// GAMMA: the re-split iteration, g_l = v_l + gamma lambda_l g_{l+1}^{old} + (1 - gamma) lambda_l g_{l+1};
// the old g_l is read before it is overwritten and kept for the next step down.
template <typename T, bool GAMMA>
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

  float carry[8], gold[8];
  load8(g + a.l_hi * layer + off, carry);
#pragma unroll
  for (int i = 0; i < 8; ++i) gold[i] = carry[i];
  const bool use_old = GAMMA && a.blk_gamma != 0.f;
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
    float gl[8];
    if (use_old) load8(g + l * layer + off, gl);     // the old g_l, for the step below
    if (GAMMA || a.lambda_tok) {
      float lam[8];
      if (a.lambda_tok) {
        load8(reinterpret_cast<const T*>(a.lambda_tok) + l * layer + off, lam);
      } else if (a.lambda) {
        load8(a.lambda + l * a.d + c0, lam);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) lam[i] = 1.f;
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (use_old) v[i] = fmaf(a.blk_gamma * lam[i], gold[i], v[i]);
        carry[i] = fmaf(a.res_scale * lam[i], carry[i], v[i]);
      }
      if (use_old) {
#pragma unroll
        for (int i = 0; i < 8; ++i) gold[i] = gl[i];
      }
    } else if (a.lambda) {
      float lam[8];
      load8(a.lambda + l * a.d + c0, lam);
#pragma unroll
      for (int i = 0; i < 8; ++i) carry[i] = fmaf(lam[i], carry[i], v[i]);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) carry[i] += v[i];
    }
    if (a.mask && l > 0) {   // the ReLU that made x_l: g_l is kept already taken through it
      const unsigned mb = a.mask[(l - 1) * vec_per_layer + idx];
#pragma unroll
      for (int i = 0; i < 8; ++i) carry[i] = ((mb >> i) & 1u) ? carry[i] : 0.f;
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
template <typename T, int NCH, bool GAMMA>
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
  float gold[GAMMA ? NCH : 1][8];   // the old g_{l+1}
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
    if (GAMMA) {
#pragma unroll
      for (int i = 0; i < 8; ++i) gold[GAMMA ? j : 0][i] = carry[j][i];
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
      if (GAMMA) {
        float lam[8], gl[8];
        load8(g + l * layer + off[j], gl);             // the old g_l, for the step below
        if (a.lambda_tok) {
          load8(reinterpret_cast<const T*>(a.lambda_tok) + l * layer + off[j], lam);
        } else if (a.lambda) {
          load8(a.lambda + l * a.d + (long)j * 512 + lane * 8, lam);
        } else {
#pragma unroll
          for (int i = 0; i < 8; ++i) lam[i] = 1.f;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          t[i] = fmaf(a.blk_gamma * lam[i], gold[GAMMA ? j : 0][i], t[i]);
          carry[j][i] = fmaf(a.res_scale * lam[i], carry[j][i], t[i]);
          gold[GAMMA ? j : 0][i] = gl[i];
        }
      } else if (a.lambda_tok) {
        float lam[8];
        load8(reinterpret_cast<const T*>(a.lambda_tok) + l * layer + off[j], lam);
#pragma unroll
        for (int i = 0; i < 8; ++i) carry[j][i] = fmaf(lam[i], carry[j][i], t[i]);
      } else if (a.lambda) {
        float lam[8];
        load8(a.lambda + l * a.d + (long)j * 512 + lane * 8, lam);
#pragma unroll
        for (int i = 0; i < 8; ++i) carry[j][i] = fmaf(lam[i], carry[j][i], t[i]);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) carry[j][i] += t[i];
      }
      if (a.mask && l > 0) {
        const unsigned mb = a.mask[((l - 1) * layer + off[j]) >> 3];
#pragma unroll
        for (int i = 0; i < 8; ++i) carry[j][i] = ((mb >> i) & 1u) ? carry[j][i] : 0.f;
      }
      store8(g + l * layer + off[j], carry[j]);
    }
  }
}

// Sum over the 64 lanes of a wave, the same value in every lane: four rotations inside each row of 16 lanes
// (DPP row_ror 8, 4, 2, 1: no LDS round trip), then the four row totals through scalar registers.
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float wave_sum_dpp(float v) {
  v += dpp_f<0x128>(v);
  v += dpp_f<0x124>(v);
  v += dpp_f<0x122>(v);
  v += dpp_f<0x121>(v);
  const int b = __builtin_bit_cast(int, v);
  const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
  const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
  const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
  const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
  return (r0 + r1) + (r2 + r3);
}

// The wave-per-row scan for rows of exactly NCH * 512 channels with the plain recurrence (no re-split, no
// mask, coefficients per channel or 1), written as a software pipeline: the loads of layer l - 1 (block input
// gradient, normalised input, coefficients, 1/rms; all as raw 16-byte vectors) are issued before the values of
// layer l are touched, without a branch between them, so that a wave always has two layers' loads in flight
// (the layer index is clamped at the bottom instead of guarded: the last stage is loaded twice).
template <typename T, int NCH, bool HAS_E, bool HAS_LAM>
__global__ __launch_bounds__(256) void scan_rows_pipe_kernel(ScanArgs a) {
  const int lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (row >= a.N) return;
  const long layer = a.N * a.d;
  T* __restrict__ g = reinterpret_cast<T*>(a.g);
  const T* __restrict__ dn = reinterpret_cast<const T*>(a.dn);
  const T* __restrict__ y = reinterpret_cast<const T*>(a.y);
  const T* __restrict__ e = reinterpret_cast<const T*>(a.e);
  const float inv_d = 1.0f / (float)a.d;
  const long off = row * a.d + lane * 8;          // chunk j: + 512 j
  const long loff = lane * 8;

  struct Stage {
    Raw8<T> v[NCH], y[NCH], e[HAS_E ? NCH : 1];
    Raw8<float> lam[HAS_LAM ? NCH : 1];
    float rinv;
  };
  auto issue = [&](Stage& st, long l) {
    const long base = l * layer + off;
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      if (NCH == 1) {     // narrow rows: measured faster with the streamed operands read non-temporally (+13 %);
        st.v[j].load_nt(dn + base + 512 * j);          // wider rows: measured slower (-3 %)
        st.y[j].load_nt(y + base + 512 * j);
        if (HAS_E) st.e[HAS_E ? j : 0].load_nt(e + base + 512 * j);
      } else {
        st.v[j].load(dn + base + 512 * j);
        st.y[j].load(y + base + 512 * j);
        if (HAS_E) st.e[HAS_E ? j : 0].load(e + base + 512 * j);
      }
      if (HAS_LAM) st.lam[HAS_LAM ? j : 0].load(a.lambda + l * a.d + loff + 512 * j);
    }
    st.rinv = a.rinv[l * a.N + row];
  };
  float carry[NCH][8];
#pragma unroll
  for (int j = 0; j < NCH; ++j) load8(g + a.l_hi * layer + off + 512 * j, carry[j]);
  auto consume = [&](const Stage& st, long l) {
    float v[NCH][8], yy[NCH][8];
    float dot = 0.f;
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      st.v[j].unpack(v[j]);
      st.y[j].unpack(yy[j]);
#pragma unroll
      for (int i = 0; i < 8; ++i) dot = fmaf(v[j][i], yy[j][i], dot);
    }
    const float m = wave_sum_dpp(dot) * inv_d;
    const float r = st.rinv;
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      float t[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) t[i] = (v[j][i] - yy[j][i] * m) * r;
      if (HAS_E) {
        float ee[8];
        st.e[HAS_E ? j : 0].unpack(ee);
#pragma unroll
        for (int i = 0; i < 8; ++i) t[i] += ee[i];
      }
      if (HAS_LAM) {
        float lam[8];
        st.lam[HAS_LAM ? j : 0].unpack(lam);
#pragma unroll
        for (int i = 0; i < 8; ++i) carry[j][i] = fmaf(lam[i], carry[j][i], t[i]);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) carry[j][i] += t[i];
      }
      store8(g + l * layer + off + 512 * j, carry[j]);
    }
  };
  Stage s0, s1;
  long l = a.l_hi - 1;
  issue(s0, l);
  while (true) {
    issue(s1, l - 1 > a.l_lo ? l - 1 : a.l_lo);
    consume(s0, l);
    if (--l < a.l_lo) break;
    issue(s0, l - 1 > a.l_lo ? l - 1 : a.l_lo);
    consume(s1, l);
    if (--l < a.l_lo) break;
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

// ---------------------------------------------------------------------------
// Chunked form for long chains (T = thousands of states, only N*d chains): the
// direct kernels above would leave most of the chip idle behind a sequential
// walk.  The chain is cut into chunks of SCAN_CHUNK states.  With the linear
// map of a chunk written  g_bottom = B + A (.) g_top  (A = product of lambda
// over the chunk, B = the chunk scanned from a zero state), three passes do:
//   reduce   every (chunk, row group, channel vector) in parallel: B
//   combine  every chain, walking the chunks from the top: the state entering
//            each chunk, cin_c = B_{c+1} + A_{c+1} (.) cin_{c+1}  (cin_top = g[l_hi])
//   apply    every (chunk, ...) in parallel again: the recurrence from cin_c,
//            writing g.
// The same operator (A1,B1) o (A2,B2) = (A1 A2, B1 + A1 B2) composes chunks as
// composes single states.  Each element is read twice and written once.
// ---------------------------------------------------------------------------
// A workgroup of 256 threads owns (chunk, 64 channels, 32 rows): thread = (row, 8
// channels).  The chunk's lambda rows for those channels are shared by all rows,
// so they are staged once in LDS (16 KB) instead of being re-read per row.
constexpr int CH_ROWS = 32;

// HAS_DN / HAS_E are compile-time so that the unrolled loop has no branches
// around its loads and several steps' loads are in flight at once.
// HAS_G: the re-split iteration's extra term gamma lambda_l (.) g_{l+1}^{old}.  A thread reads the old
// g_l of its chunk before it overwrites it; the old state above the chunk belongs to another
// workgroup's chunk, so the reduce pass (which writes nothing to g) saves it for the apply pass.
// LTOK: coefficients per token ([L,N,d], read like the other streams) instead of per channel; the
// chunk's product A is then per chain as well.
template <typename T, bool APPLY, bool HAS_DN, bool HAS_E, bool HAS_G, bool LTOK>
__global__ __launch_bounds__(256) void scan_chunk_kernel(ScanArgs a, long nchunks) {
  __shared__ float lam_s[SCAN_CHUNK][64];                  // res_scale * lambda
  __shared__ float glam_s[HAS_G ? SCAN_CHUNK : 1][64];     // blk_gamma * lambda
  const int tid = threadIdx.x;
  const long c = blockIdx.y;                 // neighbouring workgroups take neighbouring channel slabs
  const long ch0 = (long)blockIdx.x * 64;
  const long row = (long)blockIdx.z * CH_ROWS + (tid >> 3);
  const long ch = ch0 + (tid & 7) * 8;
  const long layer = a.N * a.d;
  const long l_bot = a.l_lo + c * SCAN_CHUNK;
  const long l_top = l_bot + SCAN_CHUNK < a.l_hi ? l_bot + SCAN_CHUNK : a.l_hi;
  const int steps = (int)(l_top - l_bot);
  T* __restrict__ g = reinterpret_cast<T*>(a.g);
  const T* __restrict__ dn = reinterpret_cast<const T*>(a.dn);
  const T* __restrict__ e = reinterpret_cast<const T*>(a.e);
  float* B = a.chunk_ws;                                   // [nchunks][N][d]
  float* cin = a.chunk_ws + nchunks * layer;               // [nchunks][N][d]
  float* Aout = a.chunk_ws + 2 * nchunks * layer;          // [nchunks][d], or [nchunks][N][d] with LTOK
  float* gtop = a.chunk_ws + 3 * nchunks * layer;          // [nchunks][N][d]: old g above each chunk
  const T* __restrict__ ltok = reinterpret_cast<const T*>(a.lambda_tok);

  // stage lambda[l_bot .. l_top)[ch0 .. ch0+63] (ones where there is none), scaled
  for (int i = tid; i < steps * 16; i += 256) {
    const int s = i >> 4, q = (i & 15) * 4;
    float4 v = make_float4(1.f, 1.f, 1.f, 1.f);
    if (!LTOK && a.lambda && ch0 + q < a.d) v = *reinterpret_cast<const float4*>(a.lambda + (l_bot + s) * a.d + ch0 + q);
    const float rs = a.res_scale;
    *reinterpret_cast<float4*>(&lam_s[s][q]) = make_float4(rs * v.x, rs * v.y, rs * v.z, rs * v.w);
    if (HAS_G) {
      const float bg = a.blk_gamma;
      *reinterpret_cast<float4*>(&glam_s[s][q]) = make_float4(bg * v.x, bg * v.y, bg * v.z, bg * v.w);
    }
  }
  __syncthreads();
  if (!LTOK && !APPLY && blockIdx.z == 0 && tid < 64 && ch0 + tid < a.d) {   // A = product of lambda over the chunk
    float p = 1.f;
    for (int s = 0; s < steps; ++s) p *= lam_s[s][tid];
    Aout[c * a.d + ch0 + tid] = p;
  }
  if (row >= a.N || ch >= a.d) return;

  const long off = row * a.d + ch;
  float carry[8], prod[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) { carry[i] = 0.f; prod[i] = 1.f; }
  if (APPLY) load8(cin + c * layer + off, carry);
  float gold[8];            // the old g one state up
  if (HAS_G) {
    if (APPLY) {
      load8(gtop + c * layer + off, gold);
    } else {
      load8(g + l_top * layer + off, gold);
      store8(gtop + c * layer + off, gold);
    }
  }
  // batches of 8 steps: all their loads are issued before the first value is used
  constexpr int BATCH = 8;
  for (int s0 = steps; s0 > 0; s0 -= BATCH) {
    Raw8<T> rb[BATCH], re[BATCH], rg[HAS_G ? BATCH : 1], rl[LTOK ? BATCH : 1];
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {
      const int s = s0 - 1 - j;
      if (s >= 0) {
        if (HAS_DN) rb[j].load(dn + (l_bot + s) * layer + off);
        if (HAS_E) re[j].load(e + (l_bot + s) * layer + off);
        if (HAS_G) rg[HAS_G ? j : 0].load(g + (l_bot + s) * layer + off);   // old g_l: stored to only further down
        if (LTOK) rl[LTOK ? j : 0].load(ltok + (l_bot + s) * layer + off);
      }
    }
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {
      const int s = s0 - 1 - j;
      if (s < 0) break;
      float b[8], lam[8];
      if (HAS_DN) {
        rb[j].unpack(b);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) b[i] = 0.f;
      }
      if (HAS_E) {
        float t[8];
        re[j].unpack(t);
#pragma unroll
        for (int i = 0; i < 8; ++i) b[i] += t[i];
      }
      float gl[8];
      if (LTOK) {
        float raw[8];
        rl[LTOK ? j : 0].unpack(raw);
#pragma unroll
        for (int i = 0; i < 8; ++i) { lam[i] = a.res_scale * raw[i]; gl[i] = a.blk_gamma * raw[i]; }
        if (!APPLY) {
#pragma unroll
          for (int i = 0; i < 8; ++i) prod[i] *= lam[i];
        }
      } else {
        load8(&lam_s[s][(tid & 7) * 8], lam);
        if (HAS_G) load8(&glam_s[HAS_G ? s : 0][(tid & 7) * 8], gl);
      }
      if (HAS_G) {
#pragma unroll
        for (int i = 0; i < 8; ++i) b[i] = fmaf(gl[i], gold[i], b[i]);
        rg[HAS_G ? j : 0].unpack(gold);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) carry[i] = fmaf(lam[i], carry[i], b[i]);
      if (APPLY) store8(g + (l_bot + s) * layer + off, carry);
    }
  }
  if (!APPLY) {
    store8(B + c * layer + off, carry);
    if (LTOK) store8(Aout + c * layer + off, prod);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void scan_chunk_combine_kernel(ScanArgs a, long nchunks, const float* __restrict__ A) {
  const long layer = a.N * a.d;
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= layer / 8) return;
  const long off = idx * 8;
  const long ch = off % a.d;
  const float* B = a.chunk_ws;
  float* cin = a.chunk_ws + nchunks * layer;
  float s[8];
  load8(reinterpret_cast<const T*>(a.g) + a.l_hi * layer + off, s);
  constexpr int BATCH = 8;
  for (long c0 = nchunks; c0 > 0; c0 -= BATCH) {
    Raw8<float> rb[BATCH], rp[BATCH];
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {
      const long c = c0 - 1 - j;
      if (c >= 0) { rb[j].load(B + c * layer + off); rp[j].load(a.lambda_tok ? A + c * layer + off : A + c * a.d + ch); }
    }
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {
      const long c = c0 - 1 - j;
      if (c < 0) break;
      store8(cin + c * layer + off, s);
      float b[8], p[8];
      rb[j].unpack(b);
      rp[j].unpack(p);
#pragma unroll
      for (int i = 0; i < 8; ++i) s[i] = fmaf(p[i], s[i], b[i]);
    }
  }
}

// ---------------------------------------------------------------------------
// Single-pass form for long chains (bf16 storage, plain recurrence): every element is read once and written once.
// A workgroup owns (chunk of SP_STEPS states, 4 token rows, 128 channels); a wave owns one row and a lane 2
// channels, and keeps its chunk's raw values in registers (one 4-byte load per state: a wave reads 256
// contiguous bytes).  It
//   1. scans the chunk from a zero state: the chunk's map is  g_bottom = B + A (.) g_top;
//   2. publishes (A, B) for the chunks below it (flag 1);
//   3. finds the state entering the chunk: it looks at the chunks above (64 flags at a time, one per lane of the
//      first wave) for the nearest one that has published the state X leaving it (flag 2), then applies the maps of
//      the chunks in between to X one after the other (chained decoupled look-back).  Only maps applied to a state, never maps composed with maps: whichever
//      chunk the walk starts from, the same operations produce the same bits, so runs are bitwise repeatable;
//   4. publishes its own X = B + A (.) (state entering) (flag 2) and then runs the recurrence from the entering
//      state over the registers, storing g.
// Chunks are handed out from the top of the chain down by a ticket counter in the order the workgroups start, so
// a workgroup only ever waits for workgroups that are already running: the waits end.  They are bounded all the
// same: after SP_SPIN_LIMIT polls a workgroup gives up and carries NaN on, so that a broken run is loud and
// every kernel exits.  Aggregates cross the chip through device-scope (write-through / L2-coherent) accesses:
// the writers wait for their stores to be acknowledged before the flag is raised.
// ---------------------------------------------------------------------------
constexpr int SP_STEPS = 128;         // states per chunk (64 with per-token coefficients: two raw streams)
constexpr int SP_SPIN_LIMIT = 1 << 22;

struct SpScratch {
  float* A;        // [nchunks][N][d]   product of the coefficients over the chunk, per chain
  float* B;        // [nchunks][N][d]   the chunk scanned from a zero state
  float* X;        // [nchunks][N][d]   state leaving the chunk at its bottom
  int* flags;      // [nchunks][slabs]  0: nothing, 1: (A, B) published, 2: X published (chunk 0 = top)
  int* ticket;     // next unit
};

// two floats (8-byte aligned) as one device-scope access
__device__ __forceinline__ void st_dev2(float* p, float v0, float v1) {
  const unsigned long long u = (unsigned long long)__float_as_uint(v0) | ((unsigned long long)__float_as_uint(v1) << 32);
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void ld_dev2(const float* p, float& v0, float& v1) {
  const unsigned long long u =
      __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  v0 = __uint_as_float((unsigned)u); v1 = __uint_as_float((unsigned)(u >> 32));
}

__global__ void scan_sp_init_kernel(int* flags, long n) {   // flags and the ticket (the word after them)
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) flags[i] = 0;
}

// 4 bytes at a wave-uniform 64-bit base plus a per-lane 32-bit byte offset, issued from inline assembly in the
// scalar-base address form (the compiler otherwise builds a 64-bit per-lane address for every state of the chunk
// ahead of time: two registers per pending load).  The compiler does not count this load: callers wait for it.
__device__ __forceinline__ unsigned ld_u32_s(const char* sbase, unsigned lane_off) {
  unsigned r;
  asm volatile("global_load_dword %0, %1, %2" : "=v"(r) : "v"(lane_off), "s"(sbase));
  return r;
}

typedef float float2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float2v ld_f2_s(const char* sbase, unsigned lane_off) {
  float2v r;
  asm volatile("global_load_dwordx2 %0, %1, %2" : "=v"(r) : "v"(lane_off), "s"(sbase));
  return r;
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {   // at most N vector-memory operations outstanding (N <= 63)
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
  asm volatile("" ::: "memory");
}

// The compiler does not know that the registers written by the loads above arrive later: after the wait, every
// such register passes through an empty asm statement (ordered after the wait, like every volatile asm), so
// that no use of it can be scheduled ahead of the wait.
__device__ __forceinline__ void landed(unsigned& r) { asm volatile("" : "+v"(r)); }
__device__ __forceinline__ void landed(float2v& r) { asm volatile("" : "+v"(r)); }

// Every chunk has exactly STEPS states (the launcher gives the chain's remainder to the sequential kernel).
// A workgroup is 4 waves = 4 token rows x 128 channels (a lane owns 2 channels).
// LAMK: 0 coefficients 1; 1 per channel (fp32 [L,d]): the chunk's STEPS x 128 coefficients, shared by the four rows,
// are staged once in LDS (64 KB), scaled; 2 per token: a second raw stream in registers.
constexpr int SP_ROWS = 4, SP_CH = 128;
template <int STEPS, bool HAS_SRC, int LAMK>
__global__ __launch_bounds__(256) void scan_sp_kernel(ScanArgs a, SpScratch sp, int nchunks, int slabs_ch, int slabs) {
  constexpr bool LTOK = LAMK == 2;
  extern __shared__ __attribute__((aligned(16))) float lam_s[];     // [STEPS][SP_CH] with LAMK == 1
  __shared__ int sh_unit, sh_start;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  if (tid == 0) sh_unit = atomicAdd(sp.ticket, 1);
  __syncthreads();
  const int unit = __builtin_amdgcn_readfirstlane(sh_unit);
  const int ct = unit / slabs;               // chunk, counted from the top of the chain
  const int slab = unit - ct * slabs;
  if (ct >= nchunks) return;                 // (the grid has exactly nchunks * slabs workgroups)
  const int rg = slab / slabs_ch;
  const int ch0 = (slab - rg * slabs_ch) * SP_CH;
  const int row = rg * SP_ROWS + wave;
  const int ch = ch0 + lane * 2;
  const bool valid = row < (int)a.N && ch < (int)a.d;
  const long layer = a.N * a.d;
  const long layer_b = layer * 2;                                     // bytes per state
  const long l_bot = a.l_hi - (long)(ct + 1) * STEPS;                 // chunk: states l_bot .. l_bot + STEPS - 1
  const unsigned voff = valid ? ((unsigned)row * (unsigned)a.d + (unsigned)ch) * 2u : 0u;   // lanes outside read element 0
  const char* gsrc = reinterpret_cast<const char*>(HAS_SRC ? (a.dn ? a.dn : a.e) : a.g) + l_bot * layer_b;
  const char* gtok = reinterpret_cast<const char*>(LTOK ? a.lambda_tok : a.g) + l_bot * layer_b;
  char* gout = reinterpret_cast<char*>(a.g) + l_bot * layer_b;
  const float rs = a.res_scale;

  // 1. the chunk's raw values ...
  unsigned raw[HAS_SRC ? STEPS : 1], rawl[LTOK ? STEPS : 1];
  {
    const char* p = gsrc;
    const char* q = gtok;
#pragma unroll
    for (int s = 0; s < STEPS; ++s) {
      if (HAS_SRC) { raw[HAS_SRC ? s : 0] = ld_u32_s(p, voff); p += layer_b; }
      if (LTOK) { rawl[LTOK ? s : 0] = ld_u32_s(q, voff); q += layer_b; }
    }
  }
  // ... and its coefficients into LDS (ones past the width), 4 channels per thread and pass
  if (LAMK == 1) {
    const float* lg = a.lambda + l_bot * a.d + ch0;
#pragma unroll 4
    for (int i = tid; i < STEPS * (SP_CH / 4); i += 256) {
      const int st = i / (SP_CH / 4), q = (i % (SP_CH / 4)) * 4;
      float4 v = make_float4(1.f, 1.f, 1.f, 1.f);
      if (ch0 + q < (int)a.d) v = *reinterpret_cast<const float4*>(lg + (long)st * a.d + q);
      *reinterpret_cast<float4*>(lam_s + st * SP_CH + q) = make_float4(rs * v.x, rs * v.y, rs * v.z, rs * v.w);
    }
  }
  wait_vmcnt<0>();
#pragma unroll
  for (int s = 0; s < STEPS; ++s) {
    if (HAS_SRC) landed(raw[HAS_SRC ? s : 0]);
    if (LTOK) landed(rawl[LTOK ? s : 0]);
  }
  if (LAMK == 1) __syncthreads();
  const float* lmine = lam_s + lane * 2;
  auto coeff = [&](int s, float& l0, float& l1) {
    if (LTOK) {
      const unsigned r = rawl[LTOK ? s : 0];
      l0 = rs * __uint_as_float(r << 16); l1 = rs * __uint_as_float(r & 0xFFFF0000u);
    } else if (LAMK == 1) {
      const float2 t = *reinterpret_cast<const float2*>(lmine + s * SP_CH);
      l0 = t.x; l1 = t.y;
    } else { l0 = rs; l1 = rs; }
  };
  auto value = [&](int s, float& v0, float& v1) {
    if (HAS_SRC) {
      const unsigned r = raw[HAS_SRC ? s : 0];
      v0 = __uint_as_float(r << 16); v1 = __uint_as_float(r & 0xFFFF0000u);
    } else { v0 = 0.f; v1 = 0.f; }
  };
  // 2. the chunk's map
  float B0 = 0.f, B1 = 0.f, A0 = 1.f, A1 = 1.f;
#pragma unroll
  for (int s = STEPS - 1; s >= 0; --s) {
    float l0, l1, v0, v1;
    coeff(s, l0, l1);
    value(s, v0, v1);
    B0 = fmaf(l0, B0, v0); B1 = fmaf(l1, B1, v1);
    A0 *= l0; A1 *= l1;
  }
  const long agg = (long)ct * layer + (voff >> 1);
  float S0, S1;
  if (ct == 0) {                    // the top chunk: the state above it is g[l_hi]
    const unsigned r = *reinterpret_cast<const unsigned*>(reinterpret_cast<const char*>(a.g) + a.l_hi * layer_b + voff);
    S0 = __uint_as_float(r << 16); S1 = __uint_as_float(r & 0xFFFF0000u);
  } else {
    if (valid) { st_dev2(sp.A + agg, A0, A1); st_dev2(sp.B + agg, B0, B1); }
    wait_vmcnt<0>();
    __syncthreads();
    if (tid < 64) {
      if (tid == 0)
        __hip_atomic_store(sp.flags + (long)ct * slabs + slab, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      // 3. look back: the 64 lanes of the first wave read the flags of 64 chunks above at once; the walk ends at
      // the nearest chunk that shows 2 once every chunk between it and this one shows 1
      int base = ct - 1, start = -1, spins = 0;
      while (true) {
        const int j = base - tid;
        int f = 3;                                     // above the top of the chain: nothing to wait for
        if (j >= 0) f = __hip_atomic_load(sp.flags + (long)j * slabs + slab, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned long long has2 = __ballot(f == 2), has0 = __ballot(f == 0);
        if (has2) {
          const int first = __builtin_ctzll(has2);     // nearest chunk with its leaving state published
          if ((has0 & ((1ull << first) - 1ull)) == 0) { start = base - first; break; }
        } else if (has0 == 0) {                        // 64 maps, no state yet: further up (chunk 0 shows 2 in the end)
          base -= 64;
          continue;
        }
        if (++spins > SP_SPIN_LIMIT) break;
        __builtin_amdgcn_s_sleep(4);
      }
      if (tid == 0) sh_start = start;
    }
    __syncthreads();
    const int start = __builtin_amdgcn_readfirstlane(sh_start);
    if (start < 0) {
      S0 = S1 = __builtin_nanf("");
    } else {
      const long vo = voff >> 1;
      ld_dev2(sp.X + (long)start * layer + vo, S0, S1);
      // the maps of the chunks in between, applied one after the other; four chunks' loads at a time (indices past
      // the last one are clamped and their maps replaced by the identity)
      for (int j0 = start + 1; j0 < ct; j0 += 4) {
        float a0[4], a1[4], b0[4], b1[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int j = j0 + i < ct ? j0 + i : ct - 1;
          ld_dev2(sp.A + (long)j * layer + vo, a0[i], a1[i]);
          ld_dev2(sp.B + (long)j * layer + vo, b0[i], b1[i]);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const bool on = j0 + i < ct;
          S0 = fmaf(on ? a0[i] : 1.f, S0, on ? b0[i] : 0.f);
          S1 = fmaf(on ? a1[i] : 1.f, S1, on ? b1[i] : 0.f);
        }
      }
    }
  }
  // 4. the state leaving this chunk, for the chunks below
  if (ct + 1 < nchunks) {
    if (valid) st_dev2(sp.X + agg, fmaf(A0, S0, B0), fmaf(A1, S1, B1));
    wait_vmcnt<0>();
    __syncthreads();
    if (tid == 0)
      __hip_atomic_store(sp.flags + (long)ct * slabs + slab, 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  // the recurrence from the entering state.  The raw values are unpacked again and the coefficients read from LDS
  // again (an empty asm makes them new values to the compiler: kept from the first loop they would hold two
  // more registers per state)
  wait_vmcnt<0>();
  asm volatile("" ::: "memory");
#pragma unroll
  for (int s = 0; s < STEPS; ++s) {
    if (HAS_SRC) landed(raw[HAS_SRC ? s : 0]);
    if (LTOK) landed(rawl[LTOK ? s : 0]);
  }
  {
    char* p = gout + (STEPS - 1) * layer_b;
#pragma unroll
    for (int s = STEPS - 1; s >= 0; --s) {
      float l0, l1, v0, v1;
      coeff(s, l0, l1);
      value(s, v0, v1);
      S0 = fmaf(l0, S0, v0); S1 = fmaf(l1, S1, v1);
      const unsigned o = pack_bf16x2(S0, S1);
      if (valid) asm volatile("global_store_dword %0, %1, %2" :: "v"(voff), "v"(o), "s"(p) : "memory");
      p -= layer_b;
    }
  }
}

inline bool use_chunked(long L, long N, long d, int norm_rms) {
  // long chains and too few of them to fill the chip with one thread per vector
  return !norm_rms && L >= 4 * SCAN_CHUNK && N * d / 8 < 256L * 1024;
}

template <typename T, bool APPLY, bool LTOK>
void launch_chunk_pass(const ScanArgs& a, long nchunks, dim3 grid, dim3 block, hipStream_t s) {
  const int var = (a.dn ? 1 : 0) | (a.e ? 2 : 0) | (a.blk_gamma != 0.f ? 4 : 0);
  switch (var) {
    case 0: hipLaunchKernelGGL((scan_chunk_kernel<T, APPLY, false, false, false, LTOK>), grid, block, 0, s, a, nchunks); break;
    case 1: hipLaunchKernelGGL((scan_chunk_kernel<T, APPLY, true, false, false, LTOK>), grid, block, 0, s, a, nchunks); break;
    case 2: hipLaunchKernelGGL((scan_chunk_kernel<T, APPLY, false, true, false, LTOK>), grid, block, 0, s, a, nchunks); break;
    case 3: hipLaunchKernelGGL((scan_chunk_kernel<T, APPLY, true, true, false, LTOK>), grid, block, 0, s, a, nchunks); break;
    case 4: hipLaunchKernelGGL((scan_chunk_kernel<T, APPLY, false, false, true, LTOK>), grid, block, 0, s, a, nchunks); break;
    case 5: hipLaunchKernelGGL((scan_chunk_kernel<T, APPLY, true, false, true, LTOK>), grid, block, 0, s, a, nchunks); break;
    case 6: hipLaunchKernelGGL((scan_chunk_kernel<T, APPLY, false, true, true, LTOK>), grid, block, 0, s, a, nchunks); break;
    default: hipLaunchKernelGGL((scan_chunk_kernel<T, APPLY, true, true, true, LTOK>), grid, block, 0, s, a, nchunks); break;
  }
}

template <typename T>
hipError_t launch_scan_chunked(const ScanArgs& a, hipStream_t s) {
  const long L = a.l_hi - a.l_lo;
  const long nchunks = (L + SCAN_CHUNK - 1) / SCAN_CHUNK;
  const long layer = a.N * a.d;
  float* A = a.chunk_ws + 2 * nchunks * layer;
  const dim3 block(256);
  const dim3 grid((unsigned)((a.d + 63) / 64), (unsigned)nchunks, (unsigned)((a.N + CH_ROWS - 1) / CH_ROWS));
  if (a.lambda_tok) launch_chunk_pass<T, false, true>(a, nchunks, grid, block, s);
  else launch_chunk_pass<T, false, false>(a, nchunks, grid, block, s);
  hipLaunchKernelGGL(scan_chunk_combine_kernel<T>, dim3((unsigned)((layer / 8 + 255) / 256)), block, 0, s, a, nchunks, A);
  if (a.lambda_tok) launch_chunk_pass<T, true, true>(a, nchunks, grid, block, s);
  else launch_chunk_pass<T, true, false>(a, nchunks, grid, block, s);
  return hipGetLastError();
}

inline int sp_steps(bool ltok) { return ltok ? SP_STEPS / 2 : SP_STEPS; }
inline long sp_slabs(long N, long d) { return ((N + SP_ROWS - 1) / SP_ROWS) * ((d + SP_CH - 1) / SP_CH); }

// the single-pass form covers: bf16 storage, no extra term from the old estimate (blk_gamma = 0), one value stream
inline bool sp_covers(int dtype, const ScanArgs& a) {
  return dtype == 1 && a.blk_gamma == 0.f && !a.mask && !(a.dn && a.e) && !(a.norm_rms && a.dn) && a.d % 2 == 0 &&
         a.d % 8 == 0 && a.N * a.d <= (1L << 30);     // per-lane byte offsets inside a state are 32-bit
}

hipError_t launch_scan_sp(const ScanArgs& a, hipStream_t s) {
  const bool ltok = a.lambda_tok != nullptr;
  const int steps = sp_steps(ltok);
  const long L = a.l_hi - a.l_lo;
  const long layer = a.N * a.d;
  // whole chunks only: the top L % steps states go to the sequential kernel first (it leaves g[l_hi - rem], the
  // state the chunked part starts from)
  const long rem = L % steps;
  ScanArgs top = a;
  top.l_lo = a.l_hi - rem;
  ScanArgs rest = a;
  rest.l_hi = a.l_hi - rem;
  if (rem) {
    const long vecs = layer / 8;
    const dim3 vgrid((unsigned)((vecs + 255) / 256)), vblock(256);
    if (a.res_scale != 1.f) hipLaunchKernelGGL((scan_vec_kernel<bf16_t, true>), vgrid, vblock, 0, s, top);
    else hipLaunchKernelGGL((scan_vec_kernel<bf16_t, false>), vgrid, vblock, 0, s, top);
  }
  const int nch = (int)(L / steps);
  if (nch == 0) return hipGetLastError();
  const long slabs = sp_slabs(a.N, a.d);
  if (slabs * nch > (1L << 30)) return hipErrorInvalidValue;
  SpScratch sp;
  sp.A = a.chunk_ws;
  sp.B = sp.A + (long)nch * layer;
  sp.X = sp.B + (long)nch * layer;
  sp.flags = reinterpret_cast<int*>(sp.X + (long)nch * layer);
  sp.ticket = sp.flags + (long)nch * slabs;
  const long nflags = (long)nch * slabs + 1;
  hipLaunchKernelGGL(scan_sp_init_kernel, dim3((unsigned)((nflags + 255) / 256)), dim3(256), 0, s, sp.flags, nflags);
  const dim3 grid((unsigned)(nch * slabs)), block(256);
  const int slabs_ch = (int)((a.d + SP_CH - 1) / SP_CH);
  constexpr int lam_lds = SP_STEPS * SP_CH * (int)sizeof(float);
  {   // the per-channel variants' 64 KB of dynamic LDS: raise the limit once per device
    static std::atomic<bool> done[2][64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    for (int v = 0; v < 2; ++v) {
      if (done[v][dev].load(std::memory_order_acquire)) continue;
      const void* k = v ? reinterpret_cast<const void*>(scan_sp_kernel<SP_STEPS, true, 1>)
                        : reinterpret_cast<const void*>(scan_sp_kernel<SP_STEPS, false, 1>);
      e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, lam_lds);
      if (e != hipSuccess) return e;
      done[v][dev].store(true, std::memory_order_release);
    }
  }
  const bool src = a.dn || a.e;
#define HBP_SP(STEPS_, SRC_, LAMK_)                                                                       \
  hipLaunchKernelGGL((scan_sp_kernel<STEPS_, SRC_, LAMK_>), grid, block, (LAMK_) == 1 ? lam_lds : 0, s, rest, sp, nch, \
                     slabs_ch, (int)slabs)
  if (ltok) {
    if (src) HBP_SP(SP_STEPS / 2, true, 2); else HBP_SP(SP_STEPS / 2, false, 2);
  } else if (a.lambda) {
    if (src) HBP_SP(SP_STEPS, true, 1); else HBP_SP(SP_STEPS, false, 1);
  } else {
    if (src) HBP_SP(SP_STEPS, true, 0); else HBP_SP(SP_STEPS, false, 0);
  }
#undef HBP_SP
  return hipGetLastError();
}

template <typename T>
hipError_t launch_scan_t(const ScanArgs& a, hipStream_t s) {
  if (a.l_hi <= a.l_lo) return hipSuccess;
  const bool gam = a.res_scale != 1.f || a.blk_gamma != 0.f;
  const bool rms = a.norm_rms && a.dn;
  constexpr int dtype = std::is_same<T, float>::value ? 0 : 1;
  if (a.force == 3) {
    if (!a.chunk_ws || !sp_covers(dtype, a)) return hipErrorInvalidValue;
    return launch_scan_sp(a, s);
  }
  if (a.force == 2) {
    if (!a.chunk_ws || rms || a.mask) return hipErrorInvalidValue;
    return launch_scan_chunked<T>(a, s);
  }
  if (a.force == 0 && !a.mask && a.chunk_ws && use_chunked(a.l_hi - a.l_lo, a.N, a.d, rms)) {
    // (the scratch of the three-pass form, which the callers size the workspace for, holds the single-pass form's)
    if (sp_covers(dtype, a) &&
        scan_sp_ws_bytes(a.l_hi - a.l_lo, a.N, a.d, a.lambda_tok != nullptr) <=
            scan_chunk_ws_bytes_forced(a.l_hi - a.l_lo, a.N, a.d))
      return launch_scan_sp(a, s);
    return launch_scan_chunked<T>(a, s);
  }
  if (a.norm_rms && a.dn) {
    const int nch = (int)((a.d + 511) / 512);
    dim3 grid((unsigned)((a.N + 3) / 4)), block(256);
    if (gam) {
      switch (nch) {
        case 1: hipLaunchKernelGGL((scan_rows_kernel<T, 1, true>), grid, block, 0, s, a); break;
        case 2: hipLaunchKernelGGL((scan_rows_kernel<T, 2, true>), grid, block, 0, s, a); break;
        case 3: case 4: hipLaunchKernelGGL((scan_rows_kernel<T, 4, true>), grid, block, 0, s, a); break;
        default: return hipErrorInvalidValue;   // (rejected by the caller: d > 2048)
      }
      return hipGetLastError();
    }
    if (a.d % 512 == 0 && nch <= 4 && !a.mask && !a.lambda_tok) {    // whole 512-channel chunks: the pipelined form
#define HBP_ROWS_PIPE(N_)                                                                                          \
      do {                                                                                                         \
        if (a.e && a.lambda) hipLaunchKernelGGL((scan_rows_pipe_kernel<T, N_, true, true>), grid, block, 0, s, a);      \
        else if (a.e) hipLaunchKernelGGL((scan_rows_pipe_kernel<T, N_, true, false>), grid, block, 0, s, a);            \
        else if (a.lambda) hipLaunchKernelGGL((scan_rows_pipe_kernel<T, N_, false, true>), grid, block, 0, s, a);       \
        else hipLaunchKernelGGL((scan_rows_pipe_kernel<T, N_, false, false>), grid, block, 0, s, a);                    \
      } while (0)
      switch (nch) {
        case 1: HBP_ROWS_PIPE(1); break;
        case 2: HBP_ROWS_PIPE(2); break;
        case 3: HBP_ROWS_PIPE(3); break;
        default: HBP_ROWS_PIPE(4); break;
      }
#undef HBP_ROWS_PIPE
      return hipGetLastError();
    }
    switch (nch) {
      case 1: hipLaunchKernelGGL((scan_rows_kernel<T, 1, false>), grid, block, 0, s, a); break;
      case 2: hipLaunchKernelGGL((scan_rows_kernel<T, 2, false>), grid, block, 0, s, a); break;
      case 3: hipLaunchKernelGGL((scan_rows_kernel<T, 3, false>), grid, block, 0, s, a); break;
      case 4: hipLaunchKernelGGL((scan_rows_kernel<T, 4, false>), grid, block, 0, s, a); break;
      case 5: case 6: hipLaunchKernelGGL((scan_rows_kernel<T, 6, false>), grid, block, 0, s, a); break;
      case 7: case 8: hipLaunchKernelGGL((scan_rows_kernel<T, 8, false>), grid, block, 0, s, a); break;
      default: return hipErrorInvalidValue;
    }
  } else {
    const long vecs = a.N * a.d / 8;
    const dim3 grid((unsigned)((vecs + 255) / 256)), block(256);
    if (gam) hipLaunchKernelGGL((scan_vec_kernel<T, true>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((scan_vec_kernel<T, false>), grid, block, 0, s, a);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Algorithm 1 of the paper's appendix (with the multiplier of position i being the one that carries
// i+1 to i): after sweep s, u_i holds the terms of positions i .. i + 2^(s+1) - 1 and P_i the
// product of their multipliers.  Ping-pong buffers: a sweep reads one pair and writes the other.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void hs_init_kernel(HsArgs a, float* u, float* P) {
  const long layer = a.N * a.d;
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;     // over (L+1) * layer / 8
  if (idx >= (a.L + 1) * layer / 8) return;
  const long off = idx * 8, i = off / layer, in_layer = off - i * layer;
  float v[8];
  const T* e = reinterpret_cast<const T*>(a.e);
  if (a.every_state) load8(e + off, v);
  else if (i == a.L) load8(e + in_layer, v);
  else {
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = 0.f;
  }
  store8(u + off, v);
  if (i < a.L) {
    if (a.lambda_tok) {
      float l[8];
      load8(reinterpret_cast<const T*>(a.lambda_tok) + off, l);
#pragma unroll
      for (int j = 0; j < 8; ++j) l[j] *= a.res_scale;
      store8(P + off, l);
    } else if (in_layer < a.d) {          // the first row of the layer writes the per-channel products
      float l[8];
      if (a.lambda) load8(a.lambda + i * a.d + in_layer, l);
      else {
#pragma unroll
        for (int j = 0; j < 8; ++j) l[j] = 1.f;
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) l[j] *= a.res_scale;
      store8(P + i * a.d + in_layer, l);
    }
  }
}

// u_out_i = u_in_i + P_in_i (.) u_in_{i+h}  (positions with a partner), else a copy;
// P_out_i = P_in_i P_in_{i+h}  (the per-token form here, the per-channel form in hs_p_kernel)
template <bool TOK>
__global__ __launch_bounds__(256) void hs_sweep_kernel(HsArgs a, const float* __restrict__ ui, float* __restrict__ uo,
                                                       const float* __restrict__ Pi, float* __restrict__ Po, long h) {
  const long layer = a.N * a.d;
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (a.L + 1) * layer / 8) return;
  const long off = idx * 8, i = off / layer, in_layer = off - i * layer;
  float v[8];
  load8(ui + off, v);
  if (i + h <= a.L) {
    float p[8], w[8];
    load8(ui + off + h * layer, w);
    load8(TOK ? Pi + off : Pi + i * a.d + in_layer % a.d, p);
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = fmaf(p[j], w[j], v[j]);
    if (TOK) {
      if (i + h <= a.L - 1) {
        float q[8];
        load8(Pi + off + h * layer, q);
#pragma unroll
        for (int j = 0; j < 8; ++j) p[j] *= q[j];
      }
      store8(Po + off, p);
    }
  } else if (TOK && i < a.L) {
    float p[8];
    load8(Pi + off, p);
    store8(Po + off, p);
  }
  store8(uo + off, v);
}
__global__ __launch_bounds__(256) void hs_p_kernel(const float* __restrict__ Pi, float* __restrict__ Po, long L, long d,
                                                   long h) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= L * d) return;
  const long i = idx / d;
  Po[idx] = i + h <= L - 1 ? Pi[idx] * Pi[idx + h * d] : Pi[idx];
}
template <typename T>
__global__ __launch_bounds__(256) void hs_final_kernel(HsArgs a, const float* __restrict__ u) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (a.L + 1) * a.N * a.d / 8) return;
  float v[8];
  load8(u + idx * 8, v);
  store8(reinterpret_cast<T*>(a.g) + idx * 8, v);
}

template <typename T>
hipError_t launch_hs_t(const HsArgs& a, hipStream_t s) {
  const long layer = a.N * a.d, states = (a.L + 1) * layer;
  const bool tok = a.lambda_tok != nullptr;
  const long psize = tok ? a.L * layer : a.L * a.d;
  float* u[2] = {a.ws, a.ws + states};
  float* P[2] = {a.ws + 2 * states, a.ws + 2 * states + psize};
  const dim3 block(256), grid((unsigned)((states / 8 + 255) / 256));
  hipLaunchKernelGGL(hs_init_kernel<T>, grid, block, 0, s, a, u[0], P[0]);
  int cur = 0;
  for (long h = 1; h <= a.L; h *= 2) {
    if (tok) {
      hipLaunchKernelGGL(hs_sweep_kernel<true>, grid, block, 0, s, a, u[cur], u[cur ^ 1], P[cur], P[cur ^ 1], h);
    } else {
      hipLaunchKernelGGL(hs_sweep_kernel<false>, grid, block, 0, s, a, u[cur], u[cur ^ 1], P[cur], P[cur ^ 1], h);
      hipLaunchKernelGGL(hs_p_kernel, dim3((unsigned)((psize + 255) / 256)), block, 0, s, P[cur], P[cur ^ 1], a.L, a.d, h);
    }
    cur ^= 1;
  }
  hipLaunchKernelGGL(hs_final_kernel<T>, grid, block, 0, s, a, u[cur]);
  return hipGetLastError();
}

}  // namespace

size_t hs_ws_bytes(long L, long N, long d, int lambda_kind) {
  const size_t states = (size_t)(L + 1) * N * d;
  const size_t psize = lambda_kind == 2 ? (size_t)L * N * d : (size_t)L * d;
  return (2 * states + 2 * psize) * sizeof(float);
}
hipError_t launch_scan_hillis_steele(int dtype, const HsArgs& a, hipStream_t s) {
  return dtype == 0 ? launch_hs_t<float>(a, s) : launch_hs_t<bf16_t>(a, s);
}
size_t scan_sp_ws_bytes(long L, long N, long d, int lambda_tok) {
  const long steps = lambda_tok ? SP_STEPS / 2 : SP_STEPS;
  const long nch = (L + steps - 1) / steps;
  const long slabs = ((N + 3) / 4) * ((d + 127) / 128);
  return (size_t)(3 * nch * N * d) * sizeof(float) + (size_t)(nch * slabs + 1) * sizeof(int);
}
size_t scan_chunk_ws_bytes_forced(long L, long N, long d) {
  const long nchunks = (L + SCAN_CHUNK - 1) / SCAN_CHUNK;
  return (size_t)(4 * nchunks * N * d) * sizeof(float);
}

size_t scan_chunk_ws_bytes(long L, long N, long d, int norm_rms) {
  if (!use_chunked(L, N, d, norm_rms)) return 0;
  const long nchunks = (L + SCAN_CHUNK - 1) / SCAN_CHUNK;
  return (size_t)(4 * nchunks * N * d) * sizeof(float);   // B, cin, A (per chain at most), old g above each chunk
}

namespace {
// ---------------------------------------------------------------------------
// Post-norm stacks, x_{l+1} = RMSnorm(s_l), s_l = lambda_l (.) x_l + block_l(x_l), rho_l = 1/rms(s_l):
// K_l = diag(lambda_l rho_l) and J_l = F_l - K_l (F_l the layer's Jacobian).  With the norm's backward
// P_l(G) = rho_l (G - x_{l+1} mean(G (.) x_{l+1})), the gradient with respect to the sum, the block VJP
// and the parameter gradients start from P_l(G_{l+1}); that is what g[l+1] holds (g[0] holds G_0).  With
// m_l = mean(G_{l+1} (.) x_{l+1}):  G_{l+1} J_l = P(G) . dblock/dx - lambda_l rho_l x_{l+1} m_l, so one
// iteration's scan is
//   G_l = e_l + dn_l - lambda_l rho_l x_{l+1} m_l^{old} + lambda_l rho_l G_{l+1}      (G: fp32 carry)
//   m_{l-1} = mean(G_l (.) x_l),  g[l] = rho_{l-1} (G_l - x_l m_{l-1})                (l >= 1)
// One wavefront per token row (the means are wave reductions); x_l is read once and serves both the
// projection of G_l and, one step further down, the correction term.
// With the re-split by gamma (K' = (1 - gamma) K, J' = J + gamma K) the old G_{l+1} is needed as well; it is
// recovered from what is stored, G = g/rho + x m, which turns the step into
//   G_l = e_l + dn_l + gamma lambda_l g[l+1]^{old} + (1 - gamma) lambda_l rho_l (G_{l+1} - x_{l+1} m_l^{old})
// (gamma = 1: the exact step applied to the old estimate, i.e. fixed-point iteration).  Without it the iteration
// diverges on deep post-norm stacks: J holds the norm's rank-one term of size one per layer.
// mode 0: the iteration's scan from the top (seeds g[L] from e_L, needs l_hi = L);
// mode 1: one step of exact backpropagation for layer l_lo: G_l = e_l + dn_l + lambda_l (.) g[l+1];
// mode 2: only g[L] = P_{L-1}(e_L).
// ---------------------------------------------------------------------------
template <typename T, int NCH, bool GAMMA>
__global__ __launch_bounds__(256) void scan_post_kernel(PostScanArgs a) {
  const int lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (row >= a.N) return;
  const long layer = a.N * a.d;
  T* g = reinterpret_cast<T*>(a.g);
  const T* dn = reinterpret_cast<const T*>(a.dn);
  const T* e = reinterpret_cast<const T*>(a.e);
  const T* x = reinterpret_cast<const T*>(a.x);
  const float inv_d = 1.0f / (float)a.d;
  long off[NCH];
  bool on[NCH];
  float carry[NCH][8], xn[NCH][8];
  float gold[GAMMA ? NCH : 1][8];    // the old g[l+1]
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const long c = (long)j * 512 + lane * 8;
    on[j] = c < a.d;
    off[j] = row * a.d + c;
#pragma unroll
    for (int i = 0; i < 8; ++i) { carry[j][i] = 0.f; xn[j][i] = 0.f; gold[GAMMA ? j : 0][i] = 0.f; }
  }
  const float keep = 1.f - a.gamma;
  // G (fp32, in `carry`) of state l, projected through the norm that made x_l and stored as g[l]
  auto project_store = [&](long l) {
    float dot = 0.f;
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      if (on[j]) load8(x + l * layer + off[j], xn[j]);
#pragma unroll
      for (int i = 0; i < 8; ++i) dot = fmaf(carry[j][i], xn[j][i], dot);
    }
    const float m = wave_sum(dot) * inv_d;
    const float rp = a.rho[(l - 1) * a.N + row];
    if (lane == 0) a.m_new[(l - 1) * a.N + row] = m;
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      if (!on[j]) continue;
      float o[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] = rp * (carry[j][i] - xn[j][i] * m);
      store8(g + l * layer + off[j], o);
    }
  };
  if (a.mode != 1) {   // the top: G_L = e_L
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      if (!on[j]) continue;
      load8(reinterpret_cast<const T*>(a.e_top) + off[j], carry[j]);
      if (GAMMA) load8(g + a.l_hi * layer + off[j], gold[GAMMA ? j : 0]);
    }
    project_store(a.l_hi);
    if (a.mode == 2) return;
  }
  for (long l = a.l_hi - 1; l >= a.l_lo; --l) {
    const float rl = a.rho[l * a.N + row];
    const float mo = (a.mode == 0 && dn) ? a.m_old[l * a.N + row] : 0.f;
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      if (!on[j]) continue;
      float t[8], lam[8];
      if (dn) {
        load8(dn + l * layer + off[j], t);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) t[i] = 0.f;
      }
      if (e) {
        float ee[8];
        load8(e + l * layer + off[j], ee);
#pragma unroll
        for (int i = 0; i < 8; ++i) t[i] += ee[i];
      }
      if (a.lambda) {
        load8(a.lambda + l * a.d + (long)j * 512 + lane * 8, lam);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) lam[i] = 1.f;
      }
      if (a.mode == 0 && GAMMA) {
        float gl[8];
        if (l >= 1) load8(g + l * layer + off[j], gl);     // the old g[l], for the step below
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          t[i] = fmaf(a.blk_gamma * lam[i], gold[GAMMA ? j : 0][i], t[i]);
          carry[j][i] = fmaf(keep * lam[i] * rl, carry[j][i] - xn[j][i] * mo, t[i]);
          gold[GAMMA ? j : 0][i] = gl[i];
        }
      } else if (a.mode == 0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) carry[j][i] = fmaf(keep * lam[i] * rl, carry[j][i] - xn[j][i] * mo, t[i]);
      } else {
        float gn[8];
        load8(g + (l + 1) * layer + off[j], gn);
#pragma unroll
        for (int i = 0; i < 8; ++i) carry[j][i] = fmaf(lam[i], gn[i], t[i]);
      }
    }
    if (l >= 1) {
      project_store(l);
    } else {
#pragma unroll
      for (int j = 0; j < NCH; ++j)
        if (on[j]) store8(g + off[j], carry[j]);
    }
  }
}

// The iteration's scan (mode 0) for rows of at most 2048 channels, written for memory-level parallelism: a row is
// split over WPR wavefronts of 512 channels each (a workgroup of four wavefronts holds 4 / WPR rows), so a wavefront's
// state is 8 values per lane whatever the width, and the operands of layer l - 1 (block input gradient, injected
// gradient, state, old estimate; raw 16-byte vectors) are in flight while layer l is reduced.  The row's mean is the
// sum of the wavefronts' partial sums in a fixed order, exchanged through LDS with one barrier per layer (two sets of
// slots, used in turn: a set is rewritten two barriers after it was read).  The barrier is preceded by a wait on
// LDS traffic only: the loads of the next layer stay in flight across it.  Same arithmetic as scan_post_kernel.
template <typename T, int WPR, bool GAMMA>
__global__ __launch_bounds__(256) void scan_post_split_kernel(PostScanArgs a) {
  __shared__ float red[2][4];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int part = wave % WPR;
  const long row_raw = (long)blockIdx.x * (4 / WPR) + wave / WPR;
  const bool row_ok = row_raw < a.N;                        // a spare row of the last workgroup computes row N - 1
  const long row = row_ok ? row_raw : a.N - 1;              // again and stores nothing: every wavefront meets every barrier
  const long c = (long)part * 512 + lane * 8;
  const bool on = c < a.d;
  const bool store = on && row_ok;
  const long layer = a.N * a.d;
  const long off = row * a.d + (on ? c : 0);
  T* g = reinterpret_cast<T*>(a.g);
  const T* dn = reinterpret_cast<const T*>(a.dn);
  const T* e = reinterpret_cast<const T*>(a.e);
  const T* x = reinterpret_cast<const T*>(a.x);
  const float inv_d = 1.0f / (float)a.d;
  const float keep = 1.f - a.gamma;
  int set = 0;
  auto row_sum = [&](float v) {
    v = wave_sum_dpp(v);
    if (WPR == 1) return v;
    if (lane == 0) red[set][wave] = v;
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xC07F);                     // lgkmcnt(0): the slot is written; vector loads stay in flight
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    float t = red[set][wave - part];
#pragma unroll
    for (int k = 1; k < WPR; ++k) t += red[set][wave - part + k];
    set ^= 1;
    return t;
  };
  struct Stage {
    Raw8<T> dn, e, x, g;
    Raw8<float> lam;
    float rl, mo, rp;
  };
  auto issue = [&](Stage& st, long l) {
    const long base = l * layer + off;
    if (dn) st.dn.load_nt(dn + base);
    if (e) st.e.load_nt(e + base);
    st.x.load(x + base);                                    // (read again by the next sweep's block products)
    if (GAMMA) st.g.load(g + base);
    if (a.lambda) st.lam.load(a.lambda + l * a.d + (on ? c : 0));
    st.rl = a.rho[l * a.N + row];
    st.mo = dn ? a.m_old[l * a.N + row] : 0.f;
    st.rp = a.rho[(l >= 1 ? l - 1 : 0) * a.N + row];
  };
  float carry[8], xn[8], gold[8];
  // G (fp32, in `carry`) of state l, projected through the norm that made x_l (in xn) and stored as g[l]
  auto project_store = [&](long l, float rp) {
    float dot = 0.f;
    if (on) {
#pragma unroll
      for (int i = 0; i < 8; ++i) dot = fmaf(carry[i], xn[i], dot);
    }
    const float m = row_sum(dot) * inv_d;
    if (lane == 0 && part == 0 && row_ok) a.m_new[(l - 1) * a.N + row] = m;
    float o[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = rp * (carry[i] - xn[i] * m);
    if (store) store8(g + l * layer + off, o);
  };
  {   // the top: G_L = e_L
    load8(reinterpret_cast<const T*>(a.e_top) + off, carry);
    if (GAMMA) load8(g + a.l_hi * layer + off, gold);
    load8(x + a.l_hi * layer + off, xn);
    project_store(a.l_hi, a.rho[(a.l_hi - 1) * a.N + row]);
  }
  auto consume = [&](const Stage& st, long l) {
    float t[8], lam[8];
    if (dn) {
      st.dn.unpack(t);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) t[i] = 0.f;
    }
    if (e) {
      float ee[8];
      st.e.unpack(ee);
#pragma unroll
      for (int i = 0; i < 8; ++i) t[i] += ee[i];
    }
    if (a.lambda) {
      st.lam.unpack(lam);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) lam[i] = 1.f;
    }
    const float rl = st.rl, mo = st.mo;
    if (GAMMA) {
#pragma unroll
      for (int i = 0; i < 8; ++i) t[i] = fmaf(a.blk_gamma * lam[i], gold[i], t[i]);
      st.g.unpack(gold);                                    // the old g[l], for the step below
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) carry[i] = fmaf(keep * lam[i] * rl, carry[i] - xn[i] * mo, t[i]);
    if (l >= 1) {
      st.x.unpack(xn);
      project_store(l, st.rp);
    } else if (store) {
      store8(g + off, carry);
    }
  };
  Stage s0, s1;
  long l = a.l_hi - 1;
  issue(s0, l);
  while (true) {
    issue(s1, l - 1 > a.l_lo ? l - 1 : a.l_lo);
    consume(s0, l);
    if (--l < a.l_lo) break;
    issue(s0, l - 1 > a.l_lo ? l - 1 : a.l_lo);
    consume(s1, l);
    if (--l < a.l_lo) break;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_inplace_kernel(T* x, float* rinv, long rows, long d, float eps) {
  const int lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (row >= rows) return;
  T* xr = x + row * d;
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
    store8(xr + c, v);
  }
}

// x := max(x, 0) and one mask bit per element (1 where x was positive), 8 elements per thread
template <typename T>
__global__ __launch_bounds__(256) void relu_mask_kernel(T* __restrict__ x, uint8_t* __restrict__ mask, long nvec) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= nvec) return;
  float v[8];
  load8(x + i * 8, v);
  unsigned mb = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    if (v[j] > 0.f) mb |= 1u << j; else v[j] = 0.f;
  }
  store8(x + i * 8, v);
  mask[i] = (uint8_t)mb;
}
// g := g where the mask bit is 1, else 0
template <typename T>
__global__ __launch_bounds__(256) void mask_apply_kernel(T* __restrict__ g, const uint8_t* __restrict__ mask, long nvec) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= nvec) return;
  float v[8];
  load8(g + i * 8, v);
  const unsigned mb = mask[i];
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j] = ((mb >> j) & 1u) ? v[j] : 0.f;
  store8(g + i * 8, v);
}
}  // namespace

template <typename T, bool GAMMA>
hipError_t launch_scan_post_split(const PostScanArgs& a, hipStream_t s) {
  const int nch = (int)((a.d + 511) / 512);
  const int wpr = nch <= 1 ? 1 : nch == 2 ? 2 : 4;
  const long rows_wg = 4 / wpr;
  dim3 grid((unsigned)((a.N + rows_wg - 1) / rows_wg)), block(256);
  switch (wpr) {
    case 1: hipLaunchKernelGGL((scan_post_split_kernel<T, 1, GAMMA>), grid, block, 0, s, a); break;
    case 2: hipLaunchKernelGGL((scan_post_split_kernel<T, 2, GAMMA>), grid, block, 0, s, a); break;
    default: hipLaunchKernelGGL((scan_post_split_kernel<T, 4, GAMMA>), grid, block, 0, s, a); break;
  }
  return hipGetLastError();
}

template <typename T>
hipError_t launch_scan_post_t(const PostScanArgs& a, hipStream_t s) {
  const int nch = (int)((a.d + 511) / 512);
  dim3 grid((unsigned)((a.N + 3) / 4)), block(256);
  if (a.mode == 0 && nch <= 4 && a.d % 8 == 0)
    return a.blk_gamma != 0.f ? launch_scan_post_split<T, true>(a, s) : launch_scan_post_split<T, false>(a, s);
  if (a.blk_gamma != 0.f && a.mode == 0) {
    switch (nch) {
      case 1: hipLaunchKernelGGL((scan_post_kernel<T, 1, true>), grid, block, 0, s, a); break;
      case 2: hipLaunchKernelGGL((scan_post_kernel<T, 2, true>), grid, block, 0, s, a); break;
      case 3: case 4: hipLaunchKernelGGL((scan_post_kernel<T, 4, true>), grid, block, 0, s, a); break;
      default: return hipErrorInvalidValue;   // (rejected by the caller: d > 2048)
    }
    return hipGetLastError();
  }
  switch (nch) {
    case 1: hipLaunchKernelGGL((scan_post_kernel<T, 1, false>), grid, block, 0, s, a); break;
    case 2: hipLaunchKernelGGL((scan_post_kernel<T, 2, false>), grid, block, 0, s, a); break;
    case 3: case 4: hipLaunchKernelGGL((scan_post_kernel<T, 4, false>), grid, block, 0, s, a); break;
    case 5: case 6: case 7: case 8: hipLaunchKernelGGL((scan_post_kernel<T, 8, false>), grid, block, 0, s, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_scan_post(int dtype, const PostScanArgs& a, hipStream_t s) {
  if (a.mode == 0 && a.l_hi <= a.l_lo) return hipErrorInvalidValue;
  return dtype == 0 ? launch_scan_post_t<float>(a, s) : launch_scan_post_t<bf16_t>(a, s);
}

hipError_t launch_rmsnorm_inplace(int dtype, void* x, float* rinv, long rows, long d, float eps, hipStream_t s) {
  dim3 grid((unsigned)((rows + 3) / 4)), block(256);
  if (dtype == 0) hipLaunchKernelGGL(rmsnorm_inplace_kernel<float>, grid, block, 0, s, (float*)x, rinv, rows, d, eps);
  else hipLaunchKernelGGL(rmsnorm_inplace_kernel<bf16_t>, grid, block, 0, s, (bf16_t*)x, rinv, rows, d, eps);
  return hipGetLastError();
}

hipError_t launch_relu_mask(int dtype, void* x, uint8_t* mask, long n, hipStream_t s) {
  const long nvec = n / 8;
  dim3 grid((unsigned)((nvec + 255) / 256)), block(256);
  if (dtype == 0) hipLaunchKernelGGL(relu_mask_kernel<float>, grid, block, 0, s, (float*)x, mask, nvec);
  else hipLaunchKernelGGL(relu_mask_kernel<bf16_t>, grid, block, 0, s, (bf16_t*)x, mask, nvec);
  return hipGetLastError();
}

hipError_t launch_mask_apply(int dtype, void* g, const uint8_t* mask, long n, hipStream_t s) {
  const long nvec = n / 8;
  dim3 grid((unsigned)((nvec + 255) / 256)), block(256);
  if (dtype == 0) hipLaunchKernelGGL(mask_apply_kernel<float>, grid, block, 0, s, (float*)g, mask, nvec);
  else hipLaunchKernelGGL(mask_apply_kernel<bf16_t>, grid, block, 0, s, (bf16_t*)g, mask, nvec);
  return hipGetLastError();
}

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
