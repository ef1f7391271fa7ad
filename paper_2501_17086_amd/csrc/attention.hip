// Multi-head self-attention between the two matrices of an attention sub-block (appendix, GPT-2 paragraph: every
// transformer layer is split into its self-attention and feed-forward sub-layers): forward o = softmax(q k^T / sqrt(dh)) v
// and its vector-Jacobian product  dv = P^T do,  dP = do v^T,  dS = P (.) (dP - rowsum(do (.) o)),  dq = dS k / sqrt(dh),
// dk = dS^T q / sqrt(dh).  P is never stored: the forward keeps one number per (head, query), the base-2 logarithm of
// the row's sum of exp2(s log2 e), and the backward kernels rebuild P tile by tile from q and k.
//
// bf16 storage with dh = 64 runs on the matrix cores (v_mfma_f32_32x32x16_bf16), one wavefront per tile of 32 queries
// (forward, dq) or 32 keys (dk, dv), no communication between wavefronts:
//   - the MFMA is issued so that a lane owns one query (dk/dv kernel: one key) and its 16 accumulator registers run
//     over 16 of the tile's 32 keys (queries): row statistics, the running rescale of the output and the factor
//     dP - D are per-lane scalars;
//   - the scores of a lane, rounded to bf16, are fed back as the second product's operand straight from the
//     registers: the contraction index of an MFMA is a dummy, so it is enough that the other operand is fetched
//     in the same (permuted) order of keys, which the transposing LDS read ds_read_b64_tr_b16 does from the v, k, q
//     or do tile staged once per step in the wavefront's own 4 KB of LDS;
//   - dq on one side and dk, dv on the other are two kernels that each rebuild S: seven products instead of five,
//     no atomics, results bitwise repeatable.
// Everything else (fp32 storage, other head widths) takes plain one-wavefront-per-query (per-key) kernels.
#include "hbp_common.h"

namespace hbp {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr float LOG2E = 1.4426950408889634f;

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// ------------------------------------------------------------------------------------------------------------
// plain kernels: one wavefront per query (forward, dq) or per key (dk, dv); any storage type, any head width
// ------------------------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ float dot_rows(const T* a, const T* b, int n) {
  float s = 0.f;
  for (int c = 0; c < n; ++c) s = fmaf(Elem<T>::load(a + c), Elem<T>::load(b + c), s);
  return s;
}

template <typename T>
__global__ __launch_bounds__(64) void attn_fwd_plain_kernel(AttnArgs a) {
  extern __shared__ float sh[];                  // T floats: the query's scores, then probabilities
  const int lane = threadIdx.x;
  const long p = blockIdx.x;                     // (sequence, head)
  const int i = blockIdx.y;
  const int h = (int)(p % a.heads);
  const long seq = p / a.heads;
  const long d = (long)a.heads * a.dh, ld = 3 * d;
  const T* base = reinterpret_cast<const T*>(a.qkv) + seq * a.T * ld + (long)h * a.dh;
  const T* q = base + (long)i * ld;
  const int jn = a.causal ? i + 1 : (int)a.T;
  const float c = a.scale * LOG2E;
  float m = -INFINITY;
  for (int j = lane; j < jn; j += 64) {
    const float s = c * dot_rows(q, base + (long)j * ld + d, a.dh);
    sh[j] = s;
    m = fmaxf(m, s);
  }
  m = wave_max(m);
  float sum = 0.f;
  for (int j = lane; j < jn; j += 64) {
    const float pr = exp2f(sh[j] - m);
    sh[j] = pr;
    sum += pr;
  }
  sum = wave_sum(sum);
  __syncthreads();
  T* o = reinterpret_cast<T*>(a.o) + (seq * a.T + i) * d + (long)h * a.dh;
  for (int cc = lane; cc < a.dh; cc += 64) {
    float acc = 0.f;
    for (int j = 0; j < jn; ++j) acc = fmaf(sh[j], Elem<T>::load(base + (long)j * ld + 2 * d + cc), acc);
    Elem<T>::store(o + cc, acc / sum);
  }
  if (lane == 0) a.lse[p * a.T + i] = m + log2f(sum);
}

// dq of one query; also leaves D = sum_c do[c] o[c] for the dk/dv kernel
template <typename T>
__global__ __launch_bounds__(64) void attn_bwd_q_plain_kernel(AttnArgs a) {
  extern __shared__ float sh[];                  // T floats: dS of this query
  const int lane = threadIdx.x;
  const long p = blockIdx.x;
  const int i = blockIdx.y;
  const int h = (int)(p % a.heads);
  const long seq = p / a.heads;
  const long d = (long)a.heads * a.dh, ld = 3 * d;
  const T* base = reinterpret_cast<const T*>(a.qkv) + seq * a.T * ld + (long)h * a.dh;
  const T* q = base + (long)i * ld;
  const T* dout = reinterpret_cast<const T*>(a.dout) + (seq * a.T + i) * d + (long)h * a.dh;
  const T* o = reinterpret_cast<const T*>(a.o) + (seq * a.T + i) * d + (long)h * a.dh;
  float dpart = 0.f;
  for (int cc = lane; cc < a.dh; cc += 64) dpart = fmaf(Elem<T>::load(dout + cc), Elem<T>::load(o + cc), dpart);
  const float D = wave_sum(dpart);
  const float L2 = a.lse[p * a.T + i];
  const int jn = a.causal ? i + 1 : (int)a.T;
  const float c = a.scale * LOG2E;
  for (int j = lane; j < jn; j += 64) {
    const T* k = base + (long)j * ld + d;
    const float pr = exp2f(c * dot_rows(q, k, a.dh) - L2);
    const float dp = dot_rows(dout, k + d, a.dh);
    sh[j] = pr * (dp - D);
  }
  __syncthreads();
  T* dq = reinterpret_cast<T*>(a.dqkv) + (seq * a.T + i) * ld + (long)h * a.dh;
  for (int cc = lane; cc < a.dh; cc += 64) {
    float acc = 0.f;
    for (int j = 0; j < jn; ++j) acc = fmaf(sh[j], Elem<T>::load(base + (long)j * ld + d + cc), acc);
    Elem<T>::store(dq + cc, acc * a.scale);
  }
  if (lane == 0) a.dsum[p * a.T + i] = D;
}

// dk, dv of one key (after the dq kernel: reads D)
template <typename T>
__global__ __launch_bounds__(64) void attn_bwd_kv_plain_kernel(AttnArgs a) {
  extern __shared__ float sh[];                  // 2 T floats: P and dS of this key's column
  const int lane = threadIdx.x;
  const long p = blockIdx.x;
  const int j = blockIdx.y;
  const int h = (int)(p % a.heads);
  const long seq = p / a.heads;
  const long d = (long)a.heads * a.dh, ld = 3 * d;
  const T* base = reinterpret_cast<const T*>(a.qkv) + seq * a.T * ld + (long)h * a.dh;
  const T* k = base + (long)j * ld + d;
  const T* dbase = reinterpret_cast<const T*>(a.dout) + seq * a.T * d + (long)h * a.dh;
  float* shp = sh;
  float* shs = sh + a.T;
  const int i0 = a.causal ? j : 0;
  const float c = a.scale * LOG2E;
  for (int i = i0 + lane; i < a.T; i += 64) {
    const float pr = exp2f(c * dot_rows(base + (long)i * ld, k, a.dh) - a.lse[p * a.T + i]);
    const float dp = dot_rows(dbase + (long)i * d, k + d, a.dh);
    shp[i] = pr;
    shs[i] = pr * (dp - a.dsum[p * a.T + i]);
  }
  __syncthreads();
  T* dk = reinterpret_cast<T*>(a.dqkv) + (seq * a.T + j) * ld + d + (long)h * a.dh;
  for (int cc = lane; cc < a.dh; cc += 64) {
    float ak = 0.f, av = 0.f;
    for (int i = i0; i < a.T; ++i) {
      ak = fmaf(shs[i], Elem<T>::load(base + (long)i * ld + cc), ak);
      av = fmaf(shp[i], Elem<T>::load(dbase + (long)i * d + cc), av);
    }
    Elem<T>::store(dk + cc, ak * a.scale);
    Elem<T>::store(dk + d + cc, av);
  }
}

// ------------------------------------------------------------------------------------------------------------
// matrix-core kernels: bf16, dh = 64
// ------------------------------------------------------------------------------------------------------------
// mfma(X, Y, acc): lane l, element r of acc  +=  sum_k X[8 (r/4) + 4 (l/32) + r%4][k] * Y[l % 32][k], where for one
// step of 16 k-values a lane's 8 operand elements are k = 8 (l/32) .. + 7 of row l % 32 of X and of Y.  Only the
// pairing matters: element i of lane half hh of X meets element i of lane half hh of Y.
__device__ __forceinline__ float16v mfma(bf16x8 x, bf16x8 y, float16v acc) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, acc, 0, 0, 0);
}
__device__ __forceinline__ int tile_row_of(int r, int hh) { return 8 * (r >> 2) + 4 * hh + (r & 3); }

// A wavefront's LDS tile: 32 rows x 64 bf16 (128-byte rows), 16-byte chunk c of row r at chunk c ^ ((r >> 1) & 7).
__device__ __forceinline__ int swz(int r) { return (r >> 1) & 7; }

// Lanes read what other lanes of the same wavefront wrote (and the next step overwrites what they read): the LDS
// executes a wavefront's instructions in order, so no wait is needed, only that the compiler keeps the order.
__device__ __forceinline__ void lds_handover() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// rows r0 .. r0+31 (rows at or past rmax read row rmax-1) x 64 columns from memory into the tile
__device__ __forceinline__ void tile_to_lds(const bf16_t* base, long ld, int r0, int rmax, unsigned char* tile, int lane) {
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int id = lane + 64 * u;
    const int r = id >> 3, ch = id & 7;
    int rr = r0 + r;
    rr = rr < rmax ? rr : rmax - 1;
    const uint4 v = *reinterpret_cast<const uint4*>(base + (long)rr * ld + 8 * ch);
    *reinterpret_cast<uint4*>(tile + r * 128 + ((ch ^ swz(r)) << 4)) = v;
  }
  lds_handover();
}
// operand fragment with the contraction along the tile's columns (step kk of 16 columns): lane holds row l % 32
__device__ __forceinline__ bf16x8 frag_cols_lds(const unsigned char* tile, int kk, int lane) {
  const int r = lane & 31, ch = 2 * kk + (lane >> 5);
  return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(tile + r * 128 + ((ch ^ swz(r)) << 4)));
}
// the same straight from memory
__device__ __forceinline__ bf16x8 frag_cols_mem(const bf16_t* base, long ld, int r0, int rmax, int kk, int lane) {
  int rr = r0 + (lane & 31);
  rr = rr < rmax ? rr : rmax - 1;
  return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(base + (long)rr * ld + 16 * kk + 8 * (lane >> 5)));
}
// operand fragment with the contraction along the tile's ROWS, in the order the accumulator of the first product
// holds them: lane holds column 32 m + l % 32; its element i of step t is tile row 16 t + 8 (i/4) + 4 (l/32) + i%4
// (= tile_row_of(8 t + i, l/32)).  ds_read_b64_tr_b16: within 16 lanes, lane j receives as element r' element j%4 of
// the 8 bytes addressed by lane 4 r' + j/4.
__device__ __forceinline__ bf16x8 frag_rows_lds(const unsigned char* tile, int m, int t, int lane) {
  typedef __attribute__((address_space(3))) short4v* lds_p;
  const int s = lane & 15;
  const int e = 32 * m + 16 * ((lane >> 4) & 1) + 4 * (s & 3);
  const int r_lo = 16 * t + 4 * (lane >> 5) + (s >> 2), r_hi = r_lo + 8;
  const unsigned char* p_lo = tile + r_lo * 128 + (((e >> 3) ^ swz(r_lo)) << 4) + (e & 7) * 2;
  const unsigned char* p_hi = tile + r_hi * 128 + (((e >> 3) ^ swz(r_hi)) << 4) + (e & 7) * 2;
  const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p_lo));
  const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p_hi));
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}
// 8 accumulator elements (r = 8 t .. 8 t + 7) rounded to bf16 as the second product's operand
__device__ __forceinline__ bf16x8 pack8(const float* v) {
  const uint4 w = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]),
                             pack_bf16x2(v[6], v[7]));
  return __builtin_bit_cast(bf16x8, w);
}
__device__ __forceinline__ void store4b(bf16_t* p, float a, float b, float c, float d) {
  *reinterpret_cast<uint2*>(p) = make_uint2(pack_bf16x2(a, b), pack_bf16x2(c, d));
}
// a lane's 2 x 16 results (columns 32 m + tile_row_of(r, hh)) of its row, scaled
__device__ __forceinline__ void store_row(bf16_t* row, const float16v& a0, const float16v& a1, float f, int hh) {
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    store4b(row + 8 * g + 4 * hh, a0[4 * g] * f, a0[4 * g + 1] * f, a0[4 * g + 2] * f, a0[4 * g + 3] * f);
    store4b(row + 32 + 8 * g + 4 * hh, a1[4 * g] * f, a1[4 * g + 1] * f, a1[4 * g + 2] * f, a1[4 * g + 3] * f);
  }
}

constexpr int AT_WAVES = 4;    // wavefronts (tiles) per workgroup

struct HeadPtrs {
  const bf16_t* q; const bf16_t* k; const bf16_t* v;   // row t of the head at + t * ld
  long ld, d, tok0; int h;
};
__device__ __forceinline__ HeadPtrs head_ptrs(const AttnArgs& a, long p) {
  HeadPtrs hp;
  hp.h = (int)(p % a.heads);
  const long seq = p / a.heads;
  hp.d = (long)a.heads * 64;
  hp.ld = 3 * hp.d;
  hp.tok0 = seq * a.T;
  hp.q = reinterpret_cast<const bf16_t*>(a.qkv) + hp.tok0 * hp.ld + (long)hp.h * 64;
  hp.k = hp.q + hp.d;
  hp.v = hp.k + hp.d;
  return hp;
}

template <bool CAUSAL>
__global__ __launch_bounds__(64 * AT_WAVES) void attn_fwd_mfma_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[AT_WAVES][4096];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, hh = lane >> 5;
  const int T = (int)a.T, nt = (T + 31) / 32;
  const int qt = nt - 1 - ((int)blockIdx.y * AT_WAVES + wave);     // long rows first
  if (qt < 0) return;
  const long p = blockIdx.x;
  const HeadPtrs hp = head_ptrs(a, p);
  unsigned char* tile = smem[wave];
  const int q0 = 32 * qt, qi = q0 + (lane & 31);
  const float c = a.scale * LOG2E;
  bf16x8 fq[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) fq[kk] = frag_cols_mem(hp.q, hp.ld, q0, T, kk, lane);
  float16v o0, o1;
#pragma unroll
  for (int r = 0; r < 16; ++r) { o0[r] = 0.f; o1[r] = 0.f; }
  float m = -INFINITY, l = 0.f;
  const int nkt = CAUSAL ? qt + 1 : nt;
  for (int kt = 0; kt < nkt; ++kt) {
    const int k0 = 32 * kt;
    tile_to_lds(hp.v, hp.ld, k0, T, tile, lane);
    float16v s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) s = mfma(frag_cols_mem(hp.k, hp.ld, k0, T, kk, lane), fq[kk], s);
    float sv[16];
    float tmax = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int kj = k0 + tile_row_of(r, hh);
      const bool ok = kj < T && (!CAUSAL || kj <= qi);
      sv[r] = ok ? s[r] * c : -INFINITY;
      tmax = fmaxf(tmax, sv[r]);
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    const float mn = fmaxf(m, tmax);          // finite: every tile has a key its queries may see
    const float alpha = exp2f(m - mn);
    float ps = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) { sv[r] = exp2f(sv[r] - mn); ps += sv[r]; }
    ps += __shfl_xor(ps, 32, 64);
    l = l * alpha + ps;
    m = mn;
#pragma unroll
    for (int r = 0; r < 16; ++r) { o0[r] *= alpha; o1[r] *= alpha; }
    const bf16x8 p0 = pack8(sv), p1 = pack8(sv + 8);
    o0 = mfma(frag_rows_lds(tile, 0, 0, lane), p0, o0);
    o0 = mfma(frag_rows_lds(tile, 0, 1, lane), p1, o0);
    o1 = mfma(frag_rows_lds(tile, 1, 0, lane), p0, o1);
    o1 = mfma(frag_rows_lds(tile, 1, 1, lane), p1, o1);
    lds_handover();
  }
  if (qi < T) {
    store_row(reinterpret_cast<bf16_t*>(a.o) + (hp.tok0 + qi) * hp.d + (long)hp.h * 64, o0, o1, 1.f / l, hh);
    if (hh == 0) a.lse[p * a.T + qi] = m + log2f(l);
  }
}

// D[p][t] = sum_c do[t][c] o[t][c] over the head's 64 columns: one thread per (token, head)
__global__ __launch_bounds__(256) void attn_dsum_kernel(AttnArgs a, long total) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;    // token * heads + head
  if (i >= total) return;
  const int h = (int)(i % a.heads);
  const long tok = i / a.heads;
  const long d = (long)a.heads * 64;
  const bf16_t* x = reinterpret_cast<const bf16_t*>(a.dout) + tok * d + (long)h * 64;
  const bf16_t* y = reinterpret_cast<const bf16_t*>(a.o) + tok * d + (long)h * 64;
  float acc = 0.f;
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    float xa[8], ya[8];
    load8(x + 8 * u, xa);
    load8(y + 8 * u, ya);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc = fmaf(xa[j], ya[j], acc);
  }
  const long seq = tok / a.T;
  a.dsum[(seq * a.heads + h) * a.T + tok % a.T] = acc;
}

template <bool CAUSAL>
__global__ __launch_bounds__(64 * AT_WAVES) void attn_bwd_q_mfma_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[AT_WAVES][4096];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, hh = lane >> 5;
  const int T = (int)a.T, nt = (T + 31) / 32;
  const int qt = nt - 1 - ((int)blockIdx.y * AT_WAVES + wave);
  if (qt < 0) return;
  const long p = blockIdx.x;
  const HeadPtrs hp = head_ptrs(a, p);
  const bf16_t* dob = reinterpret_cast<const bf16_t*>(a.dout) + hp.tok0 * hp.d + (long)hp.h * 64;
  unsigned char* tile = smem[wave];
  const int q0 = 32 * qt, qi = q0 + (lane & 31);
  const int qc = qi < T ? qi : T - 1;
  const float c = a.scale * LOG2E;
  const float L2 = a.lse[p * a.T + qc], D = a.dsum[p * a.T + qc];
  bf16x8 fq[4], fdo[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    fq[kk] = frag_cols_mem(hp.q, hp.ld, q0, T, kk, lane);
    fdo[kk] = frag_cols_mem(dob, hp.d, q0, T, kk, lane);
  }
  float16v dq0, dq1;
#pragma unroll
  for (int r = 0; r < 16; ++r) { dq0[r] = 0.f; dq1[r] = 0.f; }
  const int nkt = CAUSAL ? qt + 1 : nt;
  for (int kt = 0; kt < nkt; ++kt) {
    const int k0 = 32 * kt;
    tile_to_lds(hp.k, hp.ld, k0, T, tile, lane);
    float16v s, dp;
#pragma unroll
    for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      s = mfma(frag_cols_lds(tile, kk, lane), fq[kk], s);
      dp = mfma(frag_cols_mem(hp.v, hp.ld, k0, T, kk, lane), fdo[kk], dp);
    }
    float ds[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int kj = k0 + tile_row_of(r, hh);
      const bool ok = kj < T && (!CAUSAL || kj <= qi);
      const float pr = ok ? exp2f(s[r] * c - L2) : 0.f;
      ds[r] = pr * (dp[r] - D);
    }
    const bf16x8 d0 = pack8(ds), d1 = pack8(ds + 8);
    dq0 = mfma(frag_rows_lds(tile, 0, 0, lane), d0, dq0);
    dq0 = mfma(frag_rows_lds(tile, 0, 1, lane), d1, dq0);
    dq1 = mfma(frag_rows_lds(tile, 1, 0, lane), d0, dq1);
    dq1 = mfma(frag_rows_lds(tile, 1, 1, lane), d1, dq1);
    lds_handover();
  }
  if (qi < T)
    store_row(reinterpret_cast<bf16_t*>(a.dqkv) + (hp.tok0 + qi) * hp.ld + (long)hp.h * 64, dq0, dq1, a.scale, hh);
}

template <bool CAUSAL>
__global__ __launch_bounds__(64 * AT_WAVES) void attn_bwd_kv_mfma_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[AT_WAVES][2][4096];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, hh = lane >> 5;
  const int T = (int)a.T, nt = (T + 31) / 32;
  const int kt = (int)blockIdx.y * AT_WAVES + wave;                // causal: early keys see the most queries
  if (kt >= nt) return;
  const long p = blockIdx.x;
  const HeadPtrs hp = head_ptrs(a, p);
  const bf16_t* dob = reinterpret_cast<const bf16_t*>(a.dout) + hp.tok0 * hp.d + (long)hp.h * 64;
  unsigned char* tq = smem[wave][0];
  unsigned char* td = smem[wave][1];
  const int k0 = 32 * kt, kj = k0 + (lane & 31);
  const float c = a.scale * LOG2E;
  const float* lse = a.lse + p * a.T;
  const float* dsum = a.dsum + p * a.T;
  bf16x8 fk[4], fv[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    fk[kk] = frag_cols_mem(hp.k, hp.ld, k0, T, kk, lane);
    fv[kk] = frag_cols_mem(hp.v, hp.ld, k0, T, kk, lane);
  }
  float16v dk0, dk1, dv0, dv1;
#pragma unroll
  for (int r = 0; r < 16; ++r) { dk0[r] = 0.f; dk1[r] = 0.f; dv0[r] = 0.f; dv1[r] = 0.f; }
  for (int qt = CAUSAL ? kt : 0; qt < nt; ++qt) {
    const int q0 = 32 * qt;
    tile_to_lds(hp.q, hp.ld, q0, T, tq, lane);
    tile_to_lds(dob, hp.d, q0, T, td, lane);
    float16v s, dp;
#pragma unroll
    for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      s = mfma(frag_cols_lds(tq, kk, lane), fk[kk], s);
      dp = mfma(frag_cols_lds(td, kk, lane), fv[kk], dp);
    }
    float pr[16], ds[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int qi = q0 + tile_row_of(r, hh);
      const int qc = qi < T ? qi : T - 1;
      const bool ok = qi < T && kj < T && (!CAUSAL || kj <= qi);
      pr[r] = ok ? exp2f(s[r] * c - lse[qc]) : 0.f;
      ds[r] = pr[r] * (dp[r] - dsum[qc]);
    }
    const bf16x8 p0 = pack8(pr), p1 = pack8(pr + 8), d0 = pack8(ds), d1 = pack8(ds + 8);
    dv0 = mfma(frag_rows_lds(td, 0, 0, lane), p0, dv0);
    dv0 = mfma(frag_rows_lds(td, 0, 1, lane), p1, dv0);
    dv1 = mfma(frag_rows_lds(td, 1, 0, lane), p0, dv1);
    dv1 = mfma(frag_rows_lds(td, 1, 1, lane), p1, dv1);
    dk0 = mfma(frag_rows_lds(tq, 0, 0, lane), d0, dk0);
    dk0 = mfma(frag_rows_lds(tq, 0, 1, lane), d1, dk0);
    dk1 = mfma(frag_rows_lds(tq, 1, 0, lane), d0, dk1);
    dk1 = mfma(frag_rows_lds(tq, 1, 1, lane), d1, dk1);
    lds_handover();
  }
  if (kj < T) {
    bf16_t* row = reinterpret_cast<bf16_t*>(a.dqkv) + (hp.tok0 + kj) * hp.ld + hp.d + (long)hp.h * 64;
    store_row(row, dk0, dk1, a.scale, hh);
    store_row(row + hp.d, dv0, dv1, 1.f, hh);
  }
}

inline bool use_mfma(int dtype, const AttnArgs& a) { return dtype == 1 && a.dh == 64; }

}  // namespace

// the plain kernels hold a row (two rows) of T floats in LDS
bool attn_supported(int dtype, long T, int dh) {
  if (dtype == 1 && dh == 64) return T <= (1L << 20);
  return T <= 8192;
}

hipError_t launch_attn_fwd(int dtype, const AttnArgs& a, hipStream_t s) {
  const long P = a.seqs * a.heads;
  if (use_mfma(dtype, a)) {
    const dim3 grid((unsigned)P, (unsigned)(((a.T + 31) / 32 + AT_WAVES - 1) / AT_WAVES)), block(64 * AT_WAVES);
    if (a.causal) hipLaunchKernelGGL(attn_fwd_mfma_kernel<true>, grid, block, 0, s, a);
    else hipLaunchKernelGGL(attn_fwd_mfma_kernel<false>, grid, block, 0, s, a);
    return hipGetLastError();
  }
  const dim3 grid((unsigned)P, (unsigned)a.T), block(64);
  const size_t lds = (size_t)a.T * 4;
  if (dtype == 0) hipLaunchKernelGGL(attn_fwd_plain_kernel<float>, grid, block, lds, s, a);
  else hipLaunchKernelGGL(attn_fwd_plain_kernel<bf16_t>, grid, block, lds, s, a);
  return hipGetLastError();
}

hipError_t launch_attn_bwd(int dtype, const AttnArgs& a, hipStream_t s) {
  const long P = a.seqs * a.heads;
  if (use_mfma(dtype, a)) {
    const long total = a.seqs * a.T * a.heads;
    hipLaunchKernelGGL(attn_dsum_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, a, total);
    const dim3 grid((unsigned)P, (unsigned)(((a.T + 31) / 32 + AT_WAVES - 1) / AT_WAVES)), block(64 * AT_WAVES);
    if (a.causal) {
      hipLaunchKernelGGL(attn_bwd_q_mfma_kernel<true>, grid, block, 0, s, a);
      hipLaunchKernelGGL(attn_bwd_kv_mfma_kernel<true>, grid, block, 0, s, a);
    } else {
      hipLaunchKernelGGL(attn_bwd_q_mfma_kernel<false>, grid, block, 0, s, a);
      hipLaunchKernelGGL(attn_bwd_kv_mfma_kernel<false>, grid, block, 0, s, a);
    }
    return hipGetLastError();
  }
  const dim3 grid((unsigned)P, (unsigned)a.T), block(64);
  if (dtype == 0) {
    hipLaunchKernelGGL(attn_bwd_q_plain_kernel<float>, grid, block, (size_t)a.T * 4, s, a);
    hipLaunchKernelGGL(attn_bwd_kv_plain_kernel<float>, grid, block, (size_t)a.T * 8, s, a);
  } else {
    hipLaunchKernelGGL(attn_bwd_q_plain_kernel<bf16_t>, grid, block, (size_t)a.T * 4, s, a);
    hipLaunchKernelGGL(attn_bwd_kv_plain_kernel<bf16_t>, grid, block, (size_t)a.T * 8, s, a);
  }
  return hipGetLastError();
}

}  // namespace hbp
