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

#include <type_traits>

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
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }   // v_exp_f32: exp2(-inf) = 0

// A wavefront's LDS tile: 32 rows x 64 bf16 (128-byte rows), 16-byte chunk c of row r at chunk c ^ ((r >> 1) & 7).
__device__ __forceinline__ int swz(int r) { return (r >> 1) & 7; }

// Lanes read what other lanes of the same wavefront wrote (and the next step overwrites what they read): the LDS
// executes a wavefront's instructions in order, so no wait is needed, only that the compiler keeps the order.
__device__ __forceinline__ void lds_handover() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Addresses: a wavefront-uniform pointer to row 0 of the 32-row tile plus one 32-bit byte offset per lane, which is
// the same for every whole tile (LaneOffsets, computed once); a tile that runs past the last row re-reads that row
// instead (CLAMP: rows_left < 32 rows are there).
struct LaneOffsets {
  unsigned frag;       // fragment loads: row l % 32, 16 bytes at column 8 (l / 32)  (+ 32 bytes per step kk)
  unsigned tile;       // tile loads: row l / 8 (+ 8 rows per load), 16-byte chunk l % 8
  unsigned ldb;        // row stride in bytes
};
__device__ __forceinline__ LaneOffsets lane_offsets(unsigned ldb, int lane) {
  LaneOffsets o;
  o.ldb = ldb;
  o.frag = (unsigned)(lane & 31) * ldb + (unsigned)(lane >> 5) * 16u;
  o.tile = (unsigned)(lane >> 3) * ldb + (unsigned)(lane & 7) * 16u;
  return o;
}
template <bool CLAMP>
__device__ __forceinline__ void tile_to_lds(const unsigned char* base, const LaneOffsets& lo, int rows_left,
                                            unsigned char* tile, int lane) {
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int r = (lane >> 3) + 8 * u, ch = lane & 7;
    unsigned off = lo.tile + (unsigned)(8 * u) * lo.ldb;
    if (CLAMP) off = (unsigned)(r < rows_left ? r : rows_left - 1) * lo.ldb + (unsigned)ch * 16u;
    const uint4 v = *reinterpret_cast<const uint4*>(base + off);
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
template <bool CLAMP>
__device__ __forceinline__ bf16x8 frag_cols_mem(const unsigned char* base, const LaneOffsets& lo, int rows_left, int kk,
                                                int lane) {
  unsigned off = lo.frag;
  if (CLAMP) {
    const int r = lane & 31;
    off = (unsigned)(r < rows_left ? r : rows_left - 1) * lo.ldb + (unsigned)(lane >> 5) * 16u;
  }
  return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(base + off + 32u * kk));
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
__device__ __forceinline__ float dot8(bf16x8 a, bf16x8 b) {
  const uint4 x = __builtin_bit_cast(uint4, a), y = __builtin_bit_cast(uint4, b);
  const unsigned xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
  float acc = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    acc = fmaf(__uint_as_float(xs[i] << 16), __uint_as_float(ys[i] << 16), acc);
    acc = fmaf(__uint_as_float(xs[i] & 0xFFFF0000u), __uint_as_float(ys[i] & 0xFFFF0000u), acc);
  }
  return acc;
}

constexpr int AT_WAVES = 4;    // wavefronts (tiles) per workgroup

// One (sequence, head): wavefront-uniform byte pointers to row 0 of q, k, v (row stride 6 d bytes) and of the
// d-wide arrays (row stride 2 d bytes), all at the head's 64 columns.
struct Head {
  const unsigned char* q; const unsigned char* k; const unsigned char* v;
  long wide_off;         // byte offset of row 0 of the head in a [tokens, d] array
  long tok0, d, ld;
  unsigned h;
};
__device__ __forceinline__ Head head_of(const AttnArgs& a, unsigned p) {
  Head hd;
  const unsigned heads = (unsigned)a.heads;
  hd.h = p % heads;
  const unsigned seq = p / heads;
  hd.d = (long)heads * 64;
  hd.ld = 3 * hd.d;
  hd.tok0 = (long)seq * a.T;
  hd.q = reinterpret_cast<const unsigned char*>(a.qkv) + (hd.tok0 * hd.ld + (long)hd.h * 64) * 2;
  hd.k = hd.q + hd.d * 2;
  hd.v = hd.k + hd.d * 2;
  hd.wide_off = (hd.tok0 * hd.d + (long)hd.h * 64) * 2;
  return hd;
}

template <bool CAUSAL>
__global__ __launch_bounds__(64 * AT_WAVES) void attn_fwd_mfma_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[AT_WAVES][4096];
  const int lane = threadIdx.x & 63, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int T = (int)a.T, nt = (T + 31) >> 5;
  const int qt = nt - 1 - ((int)blockIdx.y * AT_WAVES + wave);     // long rows first
  if (qt < 0) return;
  const unsigned p = blockIdx.x;
  const Head hd = head_of(a, p);
  const LaneOffsets lo = lane_offsets((unsigned)(hd.ld * 2), lane);
  unsigned char* tile = smem[wave];
  const int q0 = 32 * qt, qi = q0 + (lane & 31);
  const float c = a.scale * LOG2E;
  bf16x8 fq[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) fq[kk] = frag_cols_mem<true>(hd.q + (long)q0 * lo.ldb, lo, T - q0, kk, lane);
  float16v o0, o1;
#pragma unroll
  for (int r = 0; r < 16; ++r) { o0[r] = 0.f; o1[r] = 0.f; }
  float m = -INFINITY, l = 0.f;
  const int nkt = CAUSAL ? qt + 1 : nt;
  // one tile of 32 keys; MASKED: the tile on the diagonal (causal) or the one that runs past the last key
  auto step = [&](int kt, auto masked_c) __attribute__((always_inline)) {
    constexpr bool MASKED = decltype(masked_c)::value;
    const int k0 = 32 * kt;
    const unsigned char* kb = hd.k + (long)k0 * lo.ldb;
    tile_to_lds<MASKED>(kb + hd.d * 2, lo, T - k0, tile, lane);
    float16v s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) s = mfma(frag_cols_mem<MASKED>(kb, lo, T - k0, kk, lane), fq[kk], s);
    float sv[16];
    float tmax = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      sv[r] = s[r] * c;
      if (MASKED) {
        const int kj = k0 + tile_row_of(r, hh);
        if (!(CAUSAL ? kj <= qi : kj < T)) sv[r] = -INFINITY;
      }
      tmax = fmaxf(tmax, sv[r]);
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    const float mn = fmaxf(m, tmax);          // finite: every tile has a key its queries may see
    const float alpha = fast_exp2(m - mn);
    float ps = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) { sv[r] = fast_exp2(sv[r] - mn); ps += sv[r]; }
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
  };
  const int n_plain = CAUSAL ? nkt - 1 : (T & 31 ? nkt - 1 : nkt);
  for (int kt = 0; kt < n_plain; ++kt) step(kt, std::false_type());
  if (n_plain < nkt) step(nkt - 1, std::true_type());
  if (qi < T) {
    store_row(reinterpret_cast<bf16_t*>(reinterpret_cast<unsigned char*>(a.o) + hd.wide_off) + (long)qi * hd.d, o0, o1,
              1.f / l, hh);
    if (hh == 0) a.lse[(long)p * a.T + qi] = m + log2f(l);
  }
}

// dq of a tile of 32 queries; also leaves D = rowsum(do (.) o) of its queries for the dk/dv kernel
template <bool CAUSAL>
__global__ __launch_bounds__(64 * AT_WAVES) void attn_bwd_q_mfma_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[AT_WAVES][4096];
  const int lane = threadIdx.x & 63, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int T = (int)a.T, nt = (T + 31) >> 5;
  const int qt = nt - 1 - ((int)blockIdx.y * AT_WAVES + wave);
  if (qt < 0) return;
  const unsigned p = blockIdx.x;
  const Head hd = head_of(a, p);
  const LaneOffsets lo = lane_offsets((unsigned)(hd.ld * 2), lane);
  const LaneOffsets lw = lane_offsets((unsigned)(hd.d * 2), lane);
  unsigned char* tile = smem[wave];
  const int q0 = 32 * qt, qi = q0 + (lane & 31);
  const int qc = qi < T ? qi : T - 1;
  const float c = a.scale * LOG2E;
  const float L2 = a.lse[(long)p * a.T + qc];
  bf16x8 fq[4], fdo[4];
  float D = 0.f;
  {
    const unsigned char* dob = reinterpret_cast<const unsigned char*>(a.dout) + hd.wide_off + (long)q0 * lw.ldb;
    const unsigned char* ob = reinterpret_cast<const unsigned char*>(a.o) + hd.wide_off + (long)q0 * lw.ldb;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      fq[kk] = frag_cols_mem<true>(hd.q + (long)q0 * lo.ldb, lo, T - q0, kk, lane);
      fdo[kk] = frag_cols_mem<true>(dob, lw, T - q0, kk, lane);
      D += dot8(fdo[kk], frag_cols_mem<true>(ob, lw, T - q0, kk, lane));
    }
    D += __shfl_xor(D, 32, 64);
    if (hh == 0 && qi < T) a.dsum[(long)p * a.T + qi] = D;
  }
  float16v dq0, dq1;
#pragma unroll
  for (int r = 0; r < 16; ++r) { dq0[r] = 0.f; dq1[r] = 0.f; }
  const int nkt = CAUSAL ? qt + 1 : nt;
  auto step = [&](int kt, auto masked_c) __attribute__((always_inline)) {
    constexpr bool MASKED = decltype(masked_c)::value;
    const int k0 = 32 * kt;
    const unsigned char* kb = hd.k + (long)k0 * lo.ldb;
    tile_to_lds<MASKED>(kb, lo, T - k0, tile, lane);
    float16v s, dp;
#pragma unroll
    for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = -D; }      // dp comes out as dP - D
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      s = mfma(frag_cols_lds(tile, kk, lane), fq[kk], s);
      dp = mfma(frag_cols_mem<MASKED>(kb + hd.d * 2, lo, T - k0, kk, lane), fdo[kk], dp);
    }
    float ds[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float pr = fast_exp2(fmaf(s[r], c, -L2));
      if (MASKED) {
        const int kj = k0 + tile_row_of(r, hh);
        if (!(CAUSAL ? kj <= qi : kj < T)) pr = 0.f;
      }
      ds[r] = pr * dp[r];
    }
    const bf16x8 d0 = pack8(ds), d1 = pack8(ds + 8);
    dq0 = mfma(frag_rows_lds(tile, 0, 0, lane), d0, dq0);
    dq0 = mfma(frag_rows_lds(tile, 0, 1, lane), d1, dq0);
    dq1 = mfma(frag_rows_lds(tile, 1, 0, lane), d0, dq1);
    dq1 = mfma(frag_rows_lds(tile, 1, 1, lane), d1, dq1);
    lds_handover();
  };
  const int n_plain = CAUSAL ? nkt - 1 : (T & 31 ? nkt - 1 : nkt);
  for (int kt = 0; kt < n_plain; ++kt) step(kt, std::false_type());
  if (n_plain < nkt) step(nkt - 1, std::true_type());
  if (qi < T)
    store_row(reinterpret_cast<bf16_t*>(reinterpret_cast<unsigned char*>(a.dqkv) + (hd.q - reinterpret_cast<const unsigned char*>(a.qkv))) +
                  (long)qi * hd.ld, dq0, dq1, a.scale, hh);
}

// dk, dv of a tile of 32 keys (after the dq kernel: reads D)
template <bool CAUSAL>
__global__ __launch_bounds__(64 * AT_WAVES) void attn_bwd_kv_mfma_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[AT_WAVES][2][4096];
  __shared__ __attribute__((aligned(16))) float stats[AT_WAVES][64];
  const int lane = threadIdx.x & 63, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int T = (int)a.T, nt = (T + 31) >> 5;
  const int kt = (int)blockIdx.y * AT_WAVES + wave;                // causal: early keys see the most queries
  if (kt >= nt) return;
  const unsigned p = blockIdx.x;
  const Head hd = head_of(a, p);
  const LaneOffsets lo = lane_offsets((unsigned)(hd.ld * 2), lane);
  const LaneOffsets lw = lane_offsets((unsigned)(hd.d * 2), lane);
  const unsigned char* dob = reinterpret_cast<const unsigned char*>(a.dout) + hd.wide_off;
  unsigned char* tq = smem[wave][0];
  unsigned char* td = smem[wave][1];
  float* st = stats[wave];
  const int k0 = 32 * kt, kj = k0 + (lane & 31);
  const float c = a.scale * LOG2E;
  // lanes 0..31 fetch the row statistic of query l of each tile, lanes 32..63 its D
  const float* stat_src = (hh == 0 ? a.lse : a.dsum) + (long)p * a.T;
  const float ninv_c = -1.0f / c;
  bf16x8 fk[4], fv[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    fk[kk] = frag_cols_mem<true>(hd.k + (long)k0 * lo.ldb, lo, T - k0, kk, lane);
    fv[kk] = frag_cols_mem<true>(hd.v + (long)k0 * lo.ldb, lo, T - k0, kk, lane);
  }
  float16v dk0, dk1, dv0, dv1;
#pragma unroll
  for (int r = 0; r < 16; ++r) { dk0[r] = 0.f; dk1[r] = 0.f; dv0[r] = 0.f; dv1[r] = 0.f; }
  // one tile of 32 queries; MASKED: the tile on the diagonal (causal) or the one that runs past the last query
  auto step = [&](int qt, auto masked_c) __attribute__((always_inline)) {
    constexpr bool MASKED = decltype(masked_c)::value;
    const int q0 = 32 * qt;
    {
      const int r = lane & 31;
      st[lane] = stat_src[q0 + ((!MASKED || r < T - q0) ? r : T - 1 - q0)];
    }
    tile_to_lds<MASKED>(hd.q + (long)q0 * lo.ldb, lo, T - q0, tq, lane);
    tile_to_lds<MASKED>(dob + (long)q0 * lw.ldb, lw, T - q0, td, lane);
    float16v s, dp;
#pragma unroll
    for (int g = 0; g < 4; ++g) {       // the statistics of the lane's 16 queries: rows 8 g + 4 hh .. + 3
      const float4 a4 = *reinterpret_cast<const float4*>(st + 8 * g + 4 * hh);
      const float4 d4 = *reinterpret_cast<const float4*>(st + 32 + 8 * g + 4 * hh);
      // the products start from -L2 / c and -D: they come out as (s c - L2) / c and dP - D
      s[4 * g] = a4.x * ninv_c; s[4 * g + 1] = a4.y * ninv_c; s[4 * g + 2] = a4.z * ninv_c; s[4 * g + 3] = a4.w * ninv_c;
      dp[4 * g] = -d4.x; dp[4 * g + 1] = -d4.y; dp[4 * g + 2] = -d4.z; dp[4 * g + 3] = -d4.w;
    }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      s = mfma(frag_cols_lds(tq, kk, lane), fk[kk], s);
      dp = mfma(frag_cols_lds(td, kk, lane), fv[kk], dp);
    }
    float pr[16], ds[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      pr[r] = fast_exp2(s[r] * c);
      if (MASKED) {
        const int qi = q0 + tile_row_of(r, hh);
        if (!(qi < T && (!CAUSAL || kj <= qi))) pr[r] = 0.f;
      }
      ds[r] = pr[r] * dp[r];
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
  };
  const bool ragged = (T & 31) != 0;
  int qt = CAUSAL ? kt : 0;
  if (CAUSAL) {                                  // the diagonal tile first
    step(qt, std::true_type());
    ++qt;
  }
  const int n_plain = ragged ? nt - 1 : nt;
  for (; qt < n_plain; ++qt) step(qt, std::false_type());
  if (qt < nt) step(qt, std::true_type());       // the ragged last tile (unless it was the diagonal one)
  if (kj < T) {
    bf16_t* row = reinterpret_cast<bf16_t*>(reinterpret_cast<unsigned char*>(a.dqkv) + (hd.k - reinterpret_cast<const unsigned char*>(a.qkv))) +
                  (long)kj * hd.ld;
    store_row(row, dk0, dk1, a.scale, hh);
    store_row(row + hd.d, dv0, dv1, 1.f, hh);
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
