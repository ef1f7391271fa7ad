// Multi-head self-attention between the two matrices of an attention sub-block (appendix, GPT-2 paragraph: every
// transformer layer is split into its self-attention and feed-forward sub-layers): forward o = softmax(q k^T / sqrt(dh)) v
// and its vector-Jacobian product  dv = P^T do,  dP = do v^T,  dS = P (.) (dP - rowsum(do (.) o)),  dq = dS k / sqrt(dh),
// dk = dS^T q / sqrt(dh).  P is never stored: the forward keeps one number per (head, query), the base-2 logarithm of
// the row's sum of exp2(s log2 e), and the backward kernels rebuild P tile by tile from q and k.
//
// bf16 storage with dh = 64 runs on the matrix cores (v_mfma_f32_32x32x16_bf16).  A workgroup of four wavefronts owns
// four tiles of 32 queries (forward, dq) or 32 keys (dk, dv), one per wavefront, and streams the other side's tiles
// through a ring of LDS buffers that all four read:
//   - the MFMA is issued so that a lane owns one query (dk/dv kernel: one key) and its 16 accumulator registers run
//     over 16 of the streamed tile's 32 keys (queries): row statistics, the running rescale of the output and the
//     factor dP - D are per-lane scalars (D and the row statistic enter as the accumulators' start values);
//   - the scores of a lane, rounded to bf16, are fed back as the second product's operand straight from the
//     registers: the contraction index of an MFMA is a dummy, so it is enough that the other operand is fetched
//     in the same (permuted) order of keys, which the transposing LDS read ds_read_b64_tr_b16 does from the tile;
//   - tiles reach LDS by direct copies (global_load_lds_dwordx4, no staging registers) issued three steps ahead, each
//     wavefront copying a quarter of every tile; the loop holds no other global load, so a counted s_waitcnt tells a
//     wavefront that its share of the next tile has landed, and one barrier per step completes the hand-over;
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

// Addresses: a wavefront-uniform pointer to row 0 of the 32-row tile plus one 32-bit byte offset per lane, which is
// the same for every whole tile (LaneOffsets, computed once); a tile that runs past the last row re-reads that row
// instead (CLAMP: rows_left < 32 rows are there).
struct LaneOffsets {
  unsigned frag;       // fragment loads: row l % 32, 16 bytes at column 8 (l / 32)  (+ 32 bytes per step kk)
  unsigned ldb;        // row stride in bytes
};
__device__ __forceinline__ LaneOffsets lane_offsets(unsigned ldb, int lane) {
  LaneOffsets o;
  o.ldb = ldb;
  o.frag = (unsigned)(lane & 31) * ldb + (unsigned)(lane >> 5) * 16u;
  return o;
}
// Tiles reach LDS by direct copies (global_load_lds_dwordx4: 16 bytes per lane from memory to lds_base + 16 lane,
// no staging registers), issued steps ahead into a ring of buffers.  A copy instruction fills 8 rows of the tile; the
// chunk swizzle is applied on the memory side: LDS position (row r, slot c) receives chunk c ^ swz(r) of the row.  The
// compiler sees neither the LDS write nor when it lands: a counted wait (copies_in_flight) and the workgroup's barrier
// (workgroup_handover) come before the reads.
struct CopyOffsets { unsigned o[4]; };
__device__ __forceinline__ CopyOffsets copy_offsets(unsigned ldb, int lane) {
  CopyOffsets c;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int r = 8 * u + (lane >> 3);
    c.o[u] = (unsigned)r * ldb + (unsigned)(((lane & 7) ^ swz(r)) << 4);
  }
  return c;
}
__device__ __forceinline__ void copy16_to_lds(unsigned off, const void* sbase_in, unsigned lds_base) {
  // (the base is uniform by construction; say so where the register allocator has moved it to vector registers)
  const unsigned long long b = reinterpret_cast<unsigned long long>(sbase_in);
  const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)b);
  const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(b >> 32));
  const void* sbase = reinterpret_cast<const void*>((unsigned long long)lo | ((unsigned long long)hi << 32));
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n"
               :: "v"(off), "s"(sbase), "s"(lds_base) : "memory");
}
// 4 bytes per lane from a per-lane address to lds_base + 4 lane
__device__ __forceinline__ void copy4_to_lds(const void* gptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off\n" :: "v"(gptr), "s"(lds_base) : "memory");
}
// 32 rows x 128 bytes from `base` (row 0 of the tile, wave-uniform) to the tile at LDS address lds_tile; CLAMP: only
// rows_left < 32 rows exist, the others repeat the last one
template <bool CLAMP>
__device__ __forceinline__ void copy_tile(const unsigned char* base, const CopyOffsets& co, unsigned ldb, int rows_left,
                                          unsigned lds_tile, int lane) {
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    unsigned off = co.o[u];
    if (CLAMP) {
      const int r = 8 * u + (lane >> 3);
      off = (unsigned)(r < rows_left ? r : rows_left - 1) * ldb + (unsigned)(((lane & 7) ^ swz(r)) << 4);
    }
    copy16_to_lds(off, base, lds_tile + 1024u * u);
  }
}
// this lane's byte offset into a tile for the quarter copy of wavefront w (row 8 w + l / 8, chunk (l % 8) ^ swz(row))
__device__ __forceinline__ unsigned quarter_offset(unsigned ldb, int w, int lane) {
  const int r = 8 * w + (lane >> 3);
  return (unsigned)r * ldb + (unsigned)(((lane & 7) ^ swz(r)) << 4);
}
// One wavefront's quarter of a tile copy (rows 8 w .. 8 w + 7): the four wavefronts of a workgroup fill a tile together.
template <bool CLAMP>
__device__ __forceinline__ void copy_tile_quarter(const unsigned char* base, unsigned own_off, unsigned ldb, int rows_left,
                                                  unsigned lds_tile, int w, int lane) {
  unsigned off = own_off;
  if (CLAMP) {
    const int r = 8 * w + (lane >> 3);
    off = (unsigned)(r < rows_left ? r : rows_left - 1) * ldb + (unsigned)(((lane & 7) ^ swz(r)) << 4);
  }
  copy16_to_lds(off, base, lds_tile + 1024u * (unsigned)w);
}
// at most N of this wavefront's copies still in flight (they land in issue order)
template <int N>
__device__ __forceinline__ void copies_in_flight() {
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}
// A value loaded from memory before the loop is made to arrive here.  Without this the compiler places its own counted
// waits for such loads at their first use inside the loop, and since it does not know of the direct copies, those
// waits would also drain the copies that were just issued for three steps ahead, on every step.
template <typename V>
__device__ __forceinline__ void landed(V& v) {
  asm volatile("" : "+v"(v));
}
// every wavefront of the workgroup has passed its wait: the tile is complete, and the buffer of the step before is free
__device__ __forceinline__ void workgroup_handover() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("" ::: "memory");
}
__device__ __forceinline__ unsigned lds_address(const void* p) {
  return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const unsigned char*)p;
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

constexpr int AT_WAVES = 4;    // wavefronts per workgroup: 4 tiles of 32 queries (dk/dv kernel: keys) that share the streamed tiles
constexpr int AT_NST = 4;      // stages of the ring of streamed tile pairs (8 KB each): copies run AT_NST - 1 steps ahead

// Which (sequence, head) problem and which block of AT_WAVES tiles a workgroup takes.  Consecutive workgroup ids go to
// the eight XCDs in turn, each with an L2 of its own, and all blocks of one problem stream the same k / v (q / do)
// tiles.  by_problem (large grids): the blocks of a problem get ids that land on ONE XCD, next to each other in its
// dispatch order, so they start together, stream in step and the tiles come from memory once per problem instead of
// once per block.  Otherwise (a grid of a few rounds of workgroups, where the tail decides): every problem's
// longest block first, then the next longest.  The grid holds 8 ceil(P / 8) nblk workgroups; one whose problem does
// not exist leaves at once (the whole workgroup, before any barrier).
struct BlockOf { unsigned p; int slot; bool exists; };
__device__ __forceinline__ BlockOf block_of(const AttnArgs& a, int nblk) {
  const unsigned P = (unsigned)(a.seqs * a.heads), id = blockIdx.x;
  BlockOf b;
  if (a.by_problem) {
    const unsigned xcd = id & 7u, turn = id >> 3, j = turn / (unsigned)nblk;
    b.p = xcd + 8u * j;
    b.slot = (int)(turn - j * (unsigned)nblk);
  } else {
    const unsigned Pr = (P + 7u) & ~7u;
    b.slot = (int)(id / Pr);
    b.p = id - (unsigned)b.slot * Pr;
  }
  b.exists = b.p < P;
  return b;
}
// grids from about four rounds of resident workgroups per XCD on: problem by problem
constexpr long BY_PROBLEM_FROM = 4 * 1024;
inline long attn_grid(const AttnArgs& a) {
  const long P = a.seqs * a.heads, nblk = ((a.T + 31) / 32 + AT_WAVES - 1) / AT_WAVES;
  return 8 * ((P + 7) / 8) * nblk;
}

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

// The three kernels share one shape.  A workgroup of four wavefronts owns four consecutive tiles of 32 queries
// (dk/dv kernel: keys), one per wavefront, and streams the tiles of the other side through a ring of AT_NST buffer
// pairs that all four read: at step t each wavefront waits for its own quarter of pair t, the workgroup meets at a
// barrier (pair t complete; everyone done with pair t-1), the quarter copies of pair t + AT_NST - 1 go out into the
// buffer just freed, and the wavefront computes on pair t (or skips it when the causal mask hides the whole tile from
// its rows).  No global load is issued inside the loop other than these copies, so the counted wait is exact.

template <bool CAUSAL>
__global__ __launch_bounds__(64 * AT_WAVES, 2) void attn_fwd_mfma_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(1024))) unsigned char smem[AT_NST][2][4096];   // [stage][k | v]
  const int lane = threadIdx.x & 63, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int T = (int)a.T, nt = (T + 31) >> 5;
  const int nblk = (nt + AT_WAVES - 1) / AT_WAVES;
  const BlockOf bo = block_of(a, nblk);
  if (!bo.exists) return;
  const int blk = nblk - 1 - bo.slot;                              // long rows first
  const int qt = AT_WAVES * blk + wave;
  const bool live = qt < nt;                                       // a ragged workgroup's spare wavefronts only copy
  const unsigned p = bo.p;
  const Head hd = head_of(a, p);
  const LaneOffsets lo = lane_offsets((unsigned)(hd.ld * 2), lane);
  const unsigned lds0 = lds_address(smem);
  const bool ragged = (T & 31) != 0;
  const int q0 = 32 * qt, qi = q0 + (lane & 31);
  const float c = a.scale * LOG2E;
  const int last_q = AT_WAVES * blk + AT_WAVES - 1 < nt - 1 ? AT_WAVES * blk + AT_WAVES - 1 : nt - 1;
  const int nkt = CAUSAL ? last_q + 1 : nt;                        // key tiles the workgroup streams
  const int own_nkt = CAUSAL ? qt + 1 : nt;                        // ... and those this wavefront's rows see
  const unsigned own = quarter_offset(lo.ldb, wave, lane);
  auto issue = [&](int kt) __attribute__((always_inline)) {        // this wavefront's quarters of the k and v tiles of key tile kt
    const unsigned char* kb = hd.k + (long)(32 * kt) * lo.ldb;
    const unsigned dst = lds0 + (unsigned)(kt % AT_NST) * 8192u;
    if (ragged && kt == nt - 1) {
      copy_tile_quarter<true>(kb, own, lo.ldb, T - 32 * kt, dst, wave, lane);
      copy_tile_quarter<true>(kb + hd.d * 2, own, lo.ldb, T - 32 * kt, dst + 4096u, wave, lane);
    } else {
      copy_tile_quarter<false>(kb, own, lo.ldb, 32, dst, wave, lane);
      copy_tile_quarter<false>(kb + hd.d * 2, own, lo.ldb, 32, dst + 4096u, wave, lane);
    }
  };
  for (int kt = 0; kt < AT_NST - 1 && kt < nkt; ++kt) issue(kt);
  bf16x8 fq[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) fq[kk] = frag_cols_mem<true>(hd.q + (long)(live ? q0 : 0) * lo.ldb, lo, live ? T - q0 : 1, kk, lane);
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) landed(fq[kk]);
  float16v o0, o1;
#pragma unroll
  for (int r = 0; r < 16; ++r) { o0[r] = 0.f; o1[r] = 0.f; }
  float m = -INFINITY, l = 0.f;
  // one tile of 32 keys; MASKED: the tile on the diagonal (causal) or the one that runs past the last key
  auto step = [&](int kt, auto masked_c) __attribute__((always_inline)) {
    constexpr bool MASKED = decltype(masked_c)::value;
    const int k0 = 32 * kt;
    const unsigned char* tk = smem[kt % AT_NST][0];
    const unsigned char* tv = smem[kt % AT_NST][1];
    float16v s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
    // every operand read of the step goes out here: those of the second product land while the scores are reduced
    bf16x8 fk[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) fk[kk] = frag_cols_lds(tk, kk, lane);
    const bf16x8 v00 = frag_rows_lds(tv, 0, 0, lane), v01 = frag_rows_lds(tv, 0, 1, lane);
    const bf16x8 v10 = frag_rows_lds(tv, 1, 0, lane), v11 = frag_rows_lds(tv, 1, 1, lane);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) s = mfma(fk[kk], fq[kk], s);
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
    o0 = mfma(v00, p0, o0);
    o1 = mfma(v10, p0, o1);
    o0 = mfma(v01, p1, o0);
    o1 = mfma(v11, p1, o1);
  };
  // tile kt complete and visible to the workgroup, the buffer of tile kt - 1 free and refilled
  auto advance = [&](int kt) __attribute__((always_inline)) {
    if (kt + AT_NST - 2 < nkt) copies_in_flight<2 * (AT_NST - 2)>();
    else copies_in_flight<0>();
    workgroup_handover();
    if (kt + AT_NST - 1 < nkt) issue(kt + AT_NST - 1);
  };
  // whole tiles, then the masked one, then (causal) the tiles the workgroup streams for its later rows only
  const int n_own = live ? own_nkt : 0;
  const int n_plain = CAUSAL ? n_own - 1 : (ragged ? n_own - 1 : n_own);
  int kt = 0;
  for (; kt < n_plain; ++kt) { advance(kt); step(kt, std::false_type()); }
  if (kt < n_own) { advance(kt); step(kt, std::true_type()); ++kt; }
  for (; kt < nkt; ++kt) advance(kt);
  if (live && qi < T) {
    store_row(reinterpret_cast<bf16_t*>(reinterpret_cast<unsigned char*>(a.o) + hd.wide_off) + (long)qi * hd.d, o0, o1,
              1.f / l, hh);
    if (hh == 0) a.lse[(long)p * a.T + qi] = m + log2f(l);
  }
}

// dq of four tiles of 32 queries; also leaves D = rowsum(do (.) o) of their queries for the dk/dv kernel
template <bool CAUSAL>
__global__ __launch_bounds__(64 * AT_WAVES, 2) void attn_bwd_q_mfma_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(1024))) unsigned char smem[AT_NST][2][4096];   // [stage][k | v]
  const int lane = threadIdx.x & 63, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int T = (int)a.T, nt = (T + 31) >> 5;
  const int nblk = (nt + AT_WAVES - 1) / AT_WAVES;
  const BlockOf bo = block_of(a, nblk);
  if (!bo.exists) return;
  const int blk = nblk - 1 - bo.slot;
  const int qt = AT_WAVES * blk + wave;
  const bool live = qt < nt;
  const unsigned p = bo.p;
  const Head hd = head_of(a, p);
  const LaneOffsets lo = lane_offsets((unsigned)(hd.ld * 2), lane);
  const LaneOffsets lw = lane_offsets((unsigned)(hd.d * 2), lane);
  const unsigned lds0 = lds_address(smem);
  const bool ragged = (T & 31) != 0;
  const int q0 = live ? 32 * qt : 0, qi = 32 * qt + (lane & 31);
  const int qc = qi < T ? qi : T - 1;
  const float c = a.scale * LOG2E;
  const int last_q = AT_WAVES * blk + AT_WAVES - 1 < nt - 1 ? AT_WAVES * blk + AT_WAVES - 1 : nt - 1;
  const int nkt = CAUSAL ? last_q + 1 : nt;
  const int own_nkt = CAUSAL ? qt + 1 : nt;
  const unsigned own = quarter_offset(lo.ldb, wave, lane);
  auto issue = [&](int kt) __attribute__((always_inline)) {
    const unsigned char* kb = hd.k + (long)(32 * kt) * lo.ldb;
    const unsigned dst = lds0 + (unsigned)(kt % AT_NST) * 8192u;
    if (ragged && kt == nt - 1) {
      copy_tile_quarter<true>(kb, own, lo.ldb, T - 32 * kt, dst, wave, lane);
      copy_tile_quarter<true>(kb + hd.d * 2, own, lo.ldb, T - 32 * kt, dst + 4096u, wave, lane);
    } else {
      copy_tile_quarter<false>(kb, own, lo.ldb, 32, dst, wave, lane);
      copy_tile_quarter<false>(kb + hd.d * 2, own, lo.ldb, 32, dst + 4096u, wave, lane);
    }
  };
  for (int kt = 0; kt < AT_NST - 1 && kt < nkt; ++kt) issue(kt);
  float L2 = a.lse[(long)p * a.T + qc];
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
    if (live && hh == 0 && qi < T) a.dsum[(long)p * a.T + qi] = D;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) { landed(fq[kk]); landed(fdo[kk]); }
    landed(L2);
  }
  float16v dq0, dq1;
#pragma unroll
  for (int r = 0; r < 16; ++r) { dq0[r] = 0.f; dq1[r] = 0.f; }
  auto step = [&](int kt, auto masked_c) __attribute__((always_inline)) {
    constexpr bool MASKED = decltype(masked_c)::value;
    const int k0 = 32 * kt;
    const unsigned char* tk = smem[kt % AT_NST][0];
    const unsigned char* tv = smem[kt % AT_NST][1];
    float16v s, dp;
#pragma unroll
    for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = -D; }      // dp comes out as dP - D
    // All operand reads of a phase go out before its first product (the compiler's counted waits then let the
    // products start as their operands arrive), and those of the third product while the scores become dS: a read
    // issued right before its product would expose the LDS latency a dozen times per step.
    bf16x8 fk[4], fv[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) { fk[kk] = frag_cols_lds(tk, kk, lane); fv[kk] = frag_cols_lds(tv, kk, lane); }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      s = mfma(fk[kk], fq[kk], s);
      dp = mfma(fv[kk], fdo[kk], dp);
    }
    const bf16x8 k00 = frag_rows_lds(tk, 0, 0, lane), k01 = frag_rows_lds(tk, 0, 1, lane);
    const bf16x8 k10 = frag_rows_lds(tk, 1, 0, lane), k11 = frag_rows_lds(tk, 1, 1, lane);
    __builtin_amdgcn_sched_barrier(0);
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
    __builtin_amdgcn_sched_barrier(0);
    dq0 = mfma(k00, d0, dq0);
    dq1 = mfma(k10, d0, dq1);
    dq0 = mfma(k01, d1, dq0);
    dq1 = mfma(k11, d1, dq1);
  };
  // tile kt complete and visible to the workgroup, the buffer of tile kt - 1 free and refilled
  auto advance = [&](int kt) __attribute__((always_inline)) {
    if (kt + AT_NST - 2 < nkt) copies_in_flight<2 * (AT_NST - 2)>();
    else copies_in_flight<0>();
    workgroup_handover();
    if (kt + AT_NST - 1 < nkt) issue(kt + AT_NST - 1);
  };
  // whole tiles, then the masked one, then (causal) the tiles the workgroup streams for its later rows only
  const int n_own = live ? own_nkt : 0;
  const int n_plain = CAUSAL ? n_own - 1 : (ragged ? n_own - 1 : n_own);
  int kt = 0;
  for (; kt < n_plain; ++kt) { advance(kt); step(kt, std::false_type()); }
  if (kt < n_own) { advance(kt); step(kt, std::true_type()); ++kt; }
  for (; kt < nkt; ++kt) advance(kt);
  if (live && qi < T)
    store_row(reinterpret_cast<bf16_t*>(reinterpret_cast<unsigned char*>(a.dqkv) + (hd.q - reinterpret_cast<const unsigned char*>(a.qkv))) +
                  (long)qi * hd.ld, dq0, dq1, a.scale, hh);
}

// dk, dv of four tiles of 32 keys (after the dq kernel: reads D)
template <bool CAUSAL>
__global__ __launch_bounds__(64 * AT_WAVES, 3) void attn_bwd_kv_mfma_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(1024))) unsigned char smem[AT_NST][2][4096];   // [stage][q | do]
  __shared__ __attribute__((aligned(1024))) unsigned char own[AT_WAVES][4096];      // [wave]: the v rows of the wavefront's own keys
  __shared__ __attribute__((aligned(256))) float stats[AT_WAVES][AT_NST][64];       // [wave][stage][L2 | D] (a copy per wavefront)
  const int lane = threadIdx.x & 63, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int T = (int)a.T, nt = (T + 31) >> 5;
  const BlockOf bo = block_of(a, (nt + AT_WAVES - 1) / AT_WAVES);
  if (!bo.exists) return;
  const int blk = bo.slot;                                         // causal: early keys see the most queries
  const int kt = AT_WAVES * blk + wave;
  const bool live = kt < nt;
  const unsigned p = bo.p;
  const Head hd = head_of(a, p);
  const LaneOffsets lo = lane_offsets((unsigned)(hd.ld * 2), lane);
  const unsigned ldw = (unsigned)(hd.d * 2);
  const unsigned char* dob = reinterpret_cast<const unsigned char*>(a.dout) + hd.wide_off;
  const unsigned lds0 = lds_address(smem), lds_s = lds_address(stats[wave]);
  const bool ragged = (T & 31) != 0;
  const int k0 = live ? 32 * kt : 0, kj = 32 * kt + (lane & 31);
  const float c = a.scale * LOG2E;
  const float ninv_c = -1.0f / c;
  // lanes 0..31 fetch the row statistic of query l of each tile, lanes 32..63 its D
  const float* stat_src = (hh == 0 ? a.lse : a.dsum) + (long)p * a.T;
  const int q_first = CAUSAL ? AT_WAVES * blk : 0;                 // query tiles the workgroup streams: q_first .. nt - 1
  const int own_first = CAUSAL ? kt : 0;                           // ... and the first one this wavefront's keys are seen by
  const unsigned own_q = quarter_offset(lo.ldb, wave, lane), own_d = quarter_offset(ldw, wave, lane);
  auto issue = [&](int qt) __attribute__((always_inline)) {       // quarters of the q and do tiles, and the statistics, of query tile qt
    const int q0 = 32 * qt, b = qt % AT_NST;
    const unsigned dst = lds0 + (unsigned)b * 8192u;
    int r = lane & 31;
    if (ragged && qt == nt - 1) {
      copy_tile_quarter<true>(hd.q + (long)q0 * lo.ldb, own_q, lo.ldb, T - q0, dst, wave, lane);
      copy_tile_quarter<true>(dob + (long)q0 * ldw, own_d, ldw, T - q0, dst + 4096u, wave, lane);
      r = r < T - q0 ? r : T - 1 - q0;
    } else {
      copy_tile_quarter<false>(hd.q + (long)q0 * lo.ldb, own_q, lo.ldb, 32, dst, wave, lane);
      copy_tile_quarter<false>(dob + (long)q0 * ldw, own_d, ldw, 32, dst + 4096u, wave, lane);
    }
    copy4_to_lds(stat_src + q0 + r, lds_s + (unsigned)b * 256u);
  };
  // The wavefront's own v tile stays in LDS for the whole loop (copied before the ring's first tiles, so it has landed
  // when the first of those has), its own k tile in registers: LDS and registers then both leave room for three
  // workgroups on a compute unit.
  copy_tile<true>(hd.v + (long)k0 * lo.ldb, copy_offsets(lo.ldb, lane), lo.ldb, T - k0, lds_address(own[wave]), lane);
  const unsigned char* ov = own[wave];
  for (int qt = q_first; qt < q_first + AT_NST - 1 && qt < nt; ++qt) issue(qt);
  bf16x8 fk[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) fk[kk] = frag_cols_mem<true>(hd.k + (long)k0 * lo.ldb, lo, T - k0, kk, lane);
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) landed(fk[kk]);
  float16v dk0, dk1, dv0, dv1;
#pragma unroll
  for (int r = 0; r < 16; ++r) { dk0[r] = 0.f; dk1[r] = 0.f; dv0[r] = 0.f; dv1[r] = 0.f; }
  // one tile of 32 queries; MASKED: the tile on the diagonal (causal) or the one that runs past the last query
  auto step = [&](int qt, auto masked_c) __attribute__((always_inline)) {
    constexpr bool MASKED = decltype(masked_c)::value;
    const int q0 = 32 * qt, b = qt % AT_NST;
    const unsigned char* tq = smem[b][0];
    const unsigned char* td = smem[b][1];
    const float* st = stats[wave][b];
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
      dp = mfma(frag_cols_lds(td, kk, lane), frag_cols_lds(ov, kk, lane), dp);
    }
    __builtin_amdgcn_sched_barrier(0);   // (keeps the second products' operand reads below: fewer live registers)
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
    __builtin_amdgcn_sched_barrier(0);
    dv0 = mfma(frag_rows_lds(td, 0, 0, lane), p0, dv0);
    dv0 = mfma(frag_rows_lds(td, 0, 1, lane), p1, dv0);
    dv1 = mfma(frag_rows_lds(td, 1, 0, lane), p0, dv1);
    dv1 = mfma(frag_rows_lds(td, 1, 1, lane), p1, dv1);
    dk0 = mfma(frag_rows_lds(tq, 0, 0, lane), d0, dk0);
    dk0 = mfma(frag_rows_lds(tq, 0, 1, lane), d1, dk0);
    dk1 = mfma(frag_rows_lds(tq, 1, 0, lane), d0, dk1);
    dk1 = mfma(frag_rows_lds(tq, 1, 1, lane), d1, dk1);
  };
  auto advance = [&](int qt) __attribute__((always_inline)) {
    if (qt + AT_NST - 2 < nt) copies_in_flight<3 * (AT_NST - 2)>();
    else copies_in_flight<0>();
    workgroup_handover();
    if (qt + AT_NST - 1 < nt) issue(qt + AT_NST - 1);
  };
  // (causal) the tiles streamed for the workgroup's earlier keys only, the tile on the diagonal, whole tiles, a ragged last one
  int qt = q_first;
  const int first = live ? own_first : nt;
  for (; qt < first; ++qt) advance(qt);
  if (CAUSAL && qt < nt) { advance(qt); step(qt, std::true_type()); ++qt; }
  const int plain_end = ragged ? nt - 1 : nt;
  for (; qt < plain_end; ++qt) { advance(qt); step(qt, std::false_type()); }
  if (qt < nt) { advance(qt); step(qt, std::true_type()); }
  if (live && kj < T) {
    bf16_t* row = reinterpret_cast<bf16_t*>(reinterpret_cast<unsigned char*>(a.dqkv) + (hd.k - reinterpret_cast<const unsigned char*>(a.qkv))) +
                  (long)kj * hd.ld;
    store_row(row, dk0, dk1, a.scale, hh);
    store_row(row + hd.d, dv0, dv1, 1.f, hh);
  }
}

// Backward of a whole (sequence, head) problem of at most 32 NT positions in ONE workgroup of NT wavefronts: the q, k,
// v and do tiles of the problem go to LDS once (each wavefront copies the four tiles of its own 32 positions), one
// barrier, and then nothing is streamed and nothing waited for: wavefront w first takes its positions as queries
// (dq: over the key tiles it sees) and then as keys (dk, dv: over the query tiles that see it).  Under a causal mask
// that is w + 1 and NT - w steps: every wavefront has the same number of steps.  Each tensor is read from memory once
// (the two-kernel form reads q, k, v and do twice and keeps D in memory between the kernels); the arithmetic is that
// of the two kernels, in the same order per output element.
template <bool CAUSAL, int NT>
__global__ __launch_bounds__(64 * NT, 1) void attn_bwd_short_mfma_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(1024))) unsigned char tiles[4][NT][4096];   // [q | k | v | do][tile of 32 positions]
  __shared__ __attribute__((aligned(256))) float stats[NT][64];                 // per tile: L2 of its 32 queries, then D
  const int lane = threadIdx.x & 63, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int T = (int)a.T, nt = (T + 31) >> 5;
  const bool live = wave < nt;
  const bool ragged = (T & 31) != 0;
  const unsigned p = blockIdx.x;
  const Head hd = head_of(a, p);
  const LaneOffsets lo = lane_offsets((unsigned)(hd.ld * 2), lane);
  const unsigned ldw = (unsigned)(hd.d * 2);
  const LaneOffsets lw = lane_offsets(ldw, lane);
  const unsigned char* dob = reinterpret_cast<const unsigned char*>(a.dout) + hd.wide_off;
  const unsigned char* ob = reinterpret_cast<const unsigned char*>(a.o) + hd.wide_off;
  const int r0 = live ? 32 * wave : 0;                     // (a spare wavefront repeats tile 0's loads and keeps nothing)
  const int ri = 32 * wave + (lane & 31);                  // this lane's position, as a query and as a key
  const float c = a.scale * LOG2E;
  // 1. the wavefront's four tiles (rows past the end repeat the last one), and the statistics of its queries
  if (live) {
    const CopyOffsets co = copy_offsets(lo.ldb, lane), cw = copy_offsets(ldw, lane);
    copy_tile<true>(hd.q + (long)r0 * lo.ldb, co, lo.ldb, T - r0, lds_address(tiles[0][wave]), lane);
    copy_tile<true>(hd.k + (long)r0 * lo.ldb, co, lo.ldb, T - r0, lds_address(tiles[1][wave]), lane);
    copy_tile<true>(hd.v + (long)r0 * lo.ldb, co, lo.ldb, T - r0, lds_address(tiles[2][wave]), lane);
    copy_tile<true>(dob + (long)r0 * ldw, cw, ldw, T - r0, lds_address(tiles[3][wave]), lane);
  }
  float L2 = a.lse[(long)p * a.T + (ri < T ? ri : T - 1)];
  float D = 0.f;
#pragma unroll
  for (int kk = 0; kk < 4; ++kk)
    D += dot8(frag_cols_mem<true>(dob + (long)r0 * ldw, lw, T - r0, kk, lane),
              frag_cols_mem<true>(ob + (long)r0 * ldw, lw, T - r0, kk, lane));
  D += __shfl_xor(D, 32, 64);
  if (hh == 0) { stats[wave][lane] = L2; stats[wave][32 + lane] = D; }
  copies_in_flight<0>();
  __builtin_amdgcn_s_waitcnt(0xC07F);                      // (lgkmcnt(0): the statistics are written)
  workgroup_handover();
  if (!live) return;
  // 2. the positions as queries: dq
  {
    bf16x8 fq[4], fdo[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) { fq[kk] = frag_cols_lds(tiles[0][wave], kk, lane); fdo[kk] = frag_cols_lds(tiles[3][wave], kk, lane); }
    float16v dq0, dq1;
#pragma unroll
    for (int r = 0; r < 16; ++r) { dq0[r] = 0.f; dq1[r] = 0.f; }
    auto step = [&](int kt, auto masked_c) __attribute__((always_inline)) {
      constexpr bool MASKED = decltype(masked_c)::value;
      const unsigned char* tk = tiles[1][kt];
      const unsigned char* tv = tiles[2][kt];
      float16v s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = -D; }      // dp comes out as dP - D
      bf16x8 fk[4], fv[4];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) { fk[kk] = frag_cols_lds(tk, kk, lane); fv[kk] = frag_cols_lds(tv, kk, lane); }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        s = mfma(fk[kk], fq[kk], s);
        dp = mfma(fv[kk], fdo[kk], dp);
      }
      const bf16x8 k00 = frag_rows_lds(tk, 0, 0, lane), k01 = frag_rows_lds(tk, 0, 1, lane);
      const bf16x8 k10 = frag_rows_lds(tk, 1, 0, lane), k11 = frag_rows_lds(tk, 1, 1, lane);
      __builtin_amdgcn_sched_barrier(0);
      float ds[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float pr = fast_exp2(fmaf(s[r], c, -L2));
        if (MASKED) {
          const int kj = 32 * kt + tile_row_of(r, hh);
          if (!(CAUSAL ? kj <= ri : kj < T)) pr = 0.f;
        }
        ds[r] = pr * dp[r];
      }
      const bf16x8 d0 = pack8(ds), d1 = pack8(ds + 8);
      __builtin_amdgcn_sched_barrier(0);
      dq0 = mfma(k00, d0, dq0);
      dq1 = mfma(k10, d0, dq1);
      dq0 = mfma(k01, d1, dq0);
      dq1 = mfma(k11, d1, dq1);
    };
    const int n_own = CAUSAL ? wave + 1 : nt;
    const int n_plain = CAUSAL ? n_own - 1 : (ragged ? n_own - 1 : n_own);
    int kt = 0;
    for (; kt < n_plain; ++kt) step(kt, std::false_type());
    if (kt < n_own) step(kt, std::true_type());
    if (ri < T)
      store_row(reinterpret_cast<bf16_t*>(reinterpret_cast<unsigned char*>(a.dqkv) + (hd.q - reinterpret_cast<const unsigned char*>(a.qkv))) +
                    (long)ri * hd.ld, dq0, dq1, a.scale, hh);
  }
  // 3. the positions as keys: dk, dv
  {
    bf16x8 fk[4], fv[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) { fk[kk] = frag_cols_lds(tiles[1][wave], kk, lane); fv[kk] = frag_cols_lds(tiles[2][wave], kk, lane); }
    float16v dk0, dk1, dv0, dv1;
#pragma unroll
    for (int r = 0; r < 16; ++r) { dk0[r] = 0.f; dk1[r] = 0.f; dv0[r] = 0.f; dv1[r] = 0.f; }
    const float ninv_c = -1.0f / c;
    auto step = [&](int qt, auto masked_c) __attribute__((always_inline)) {
      constexpr bool MASKED = decltype(masked_c)::value;
      const unsigned char* tq = tiles[0][qt];
      const unsigned char* td = tiles[3][qt];
      const float* st = stats[qt];
      float16v s, dp;
#pragma unroll
      for (int g = 0; g < 4; ++g) {       // the statistics of the lane's 16 queries: rows 8 g + 4 hh .. + 3
        const float4 a4 = *reinterpret_cast<const float4*>(st + 8 * g + 4 * hh);
        const float4 d4 = *reinterpret_cast<const float4*>(st + 32 + 8 * g + 4 * hh);
        // the products start from -L2 / c and -D: they come out as (s c - L2) / c and dP - D
        s[4 * g] = a4.x * ninv_c; s[4 * g + 1] = a4.y * ninv_c; s[4 * g + 2] = a4.z * ninv_c; s[4 * g + 3] = a4.w * ninv_c;
        dp[4 * g] = -d4.x; dp[4 * g + 1] = -d4.y; dp[4 * g + 2] = -d4.z; dp[4 * g + 3] = -d4.w;
      }
      bf16x8 fqs[4], fds[4];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) { fqs[kk] = frag_cols_lds(tq, kk, lane); fds[kk] = frag_cols_lds(td, kk, lane); }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        s = mfma(fqs[kk], fk[kk], s);
        dp = mfma(fds[kk], fv[kk], dp);
      }
      const bf16x8 t00 = frag_rows_lds(td, 0, 0, lane), t01 = frag_rows_lds(td, 0, 1, lane);
      const bf16x8 t10 = frag_rows_lds(td, 1, 0, lane), t11 = frag_rows_lds(td, 1, 1, lane);
      const bf16x8 u00 = frag_rows_lds(tq, 0, 0, lane), u01 = frag_rows_lds(tq, 0, 1, lane);
      const bf16x8 u10 = frag_rows_lds(tq, 1, 0, lane), u11 = frag_rows_lds(tq, 1, 1, lane);
      __builtin_amdgcn_sched_barrier(0);
      float pr[16], ds[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        pr[r] = fast_exp2(s[r] * c);
        if (MASKED) {
          const int qi = 32 * qt + tile_row_of(r, hh);
          if (!(qi < T && (!CAUSAL || ri <= qi))) pr[r] = 0.f;
        }
        ds[r] = pr[r] * dp[r];
      }
      const bf16x8 p0 = pack8(pr), p1 = pack8(pr + 8), d0 = pack8(ds), d1 = pack8(ds + 8);
      __builtin_amdgcn_sched_barrier(0);
      dv0 = mfma(t00, p0, dv0);
      dv1 = mfma(t10, p0, dv1);
      dk0 = mfma(u00, d0, dk0);
      dk1 = mfma(u10, d0, dk1);
      dv0 = mfma(t01, p1, dv0);
      dv1 = mfma(t11, p1, dv1);
      dk0 = mfma(u01, d1, dk0);
      dk1 = mfma(u11, d1, dk1);
    };
    int qt = CAUSAL ? wave : 0;
    if (CAUSAL) { step(qt, std::true_type()); ++qt; }
    const int plain_end = ragged ? nt - 1 : nt;
    for (; qt < plain_end; ++qt) step(qt, std::false_type());
    if (qt < nt) step(qt, std::true_type());
    if (ri < T) {
      bf16_t* row = reinterpret_cast<bf16_t*>(reinterpret_cast<unsigned char*>(a.dqkv) + (hd.k - reinterpret_cast<const unsigned char*>(a.qkv))) +
                    (long)ri * hd.ld;
      store_row(row, dk0, dk1, a.scale, hh);
      store_row(row + hd.d, dv0, dv1, 1.f, hh);
    }
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
    if (attn_grid(a) > 0x7fffffffL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)attn_grid(a)), block(64 * AT_WAVES);
    AttnArgs m = a;
    m.by_problem = attn_grid(a) >= BY_PROBLEM_FROM;
    if (a.causal) hipLaunchKernelGGL(attn_fwd_mfma_kernel<true>, grid, block, 0, s, m);
    else hipLaunchKernelGGL(attn_fwd_mfma_kernel<false>, grid, block, 0, s, m);
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
    if (a.T <= 256) {        // a whole problem per workgroup
      if (P > 0x7fffffffL) return hipErrorInvalidValue;
      const dim3 grid((unsigned)P);
      if (a.T <= 128) {
        if (a.causal) hipLaunchKernelGGL((attn_bwd_short_mfma_kernel<true, 4>), grid, dim3(256), 0, s, a);
        else hipLaunchKernelGGL((attn_bwd_short_mfma_kernel<false, 4>), grid, dim3(256), 0, s, a);
      } else {
        if (a.causal) hipLaunchKernelGGL((attn_bwd_short_mfma_kernel<true, 8>), grid, dim3(512), 0, s, a);
        else hipLaunchKernelGGL((attn_bwd_short_mfma_kernel<false, 8>), grid, dim3(512), 0, s, a);
      }
      return hipGetLastError();
    }
    if (attn_grid(a) > 0x7fffffffL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)attn_grid(a)), block(64 * AT_WAVES);
    // dq is bound by its tile stream and gains from one XCD per problem; dk/dv is bound by its arithmetic and by the
    // tail, and keeps the longest-first order (by_problem = 0 as the caller leaves it)
    AttnArgs m = a;
    m.by_problem = attn_grid(a) >= BY_PROBLEM_FROM;
    if (a.causal) {
      hipLaunchKernelGGL(attn_bwd_q_mfma_kernel<true>, grid, block, 0, s, m);
      hipLaunchKernelGGL(attn_bwd_kv_mfma_kernel<true>, grid, block, 0, s, a);
    } else {
      hipLaunchKernelGGL(attn_bwd_q_mfma_kernel<false>, grid, block, 0, s, m);
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
