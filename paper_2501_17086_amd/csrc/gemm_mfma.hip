// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32
// accumulate) for the VJP and parameter-gradient contractions.
//
// Shape of the kernels
//   workgroup   8 wavefronts, output tile 256 x 256, one workgroup per CU; a
//               wavefront owns 128 x 64 = 4 x 2 MFMA blocks of 32 x 32 (128
//               accumulator registers per lane).  The 256 x 256 tile keeps the
//               global -> LDS stream, which is what bounds the kernel (measured:
//               the copies alone take 0.6 of the time the MFMAs alone take),
//               at 128 flop per byte copied.
//   persistent  one workgroup per CU walks a list of tiles.  The K slices of all
//               its tiles form one stream through a ring of 4 LDS stages, so the
//               first slices of the next tile are already in flight while the
//               current tile's epilogue runs: no per-tile fill latency.
//   two phases  the wavefronts form two groups of four (one wavefront of each
//               group per SIMD).  A wavefront alternates between a load phase
//               (issue its share of the global -> LDS copy of the slice three
//               ahead, read all fragments of the current slice from LDS, store
//               a finished tile) and a compute phase (16 MFMAs back to back
//               at raised priority), with a workgroup barrier after each
//               phase.  The second group runs one barrier behind the first, so
//               on every SIMD one wavefront multiplies while the other one
//               loads: the LDS latency is paid once per slice, in bulk, and
//               hidden behind the other group's MFMAs.  A wavefront issues at
//               most one instruction every four cycles, so the load phase has to
//               be short in instructions to fit under the 512 MFMA cycles of the
//               other group: the lean kernel's is about 50.
//   K pipeline  slices of 32 (32 KB per stage); a slice is copied global -> LDS
//               directly (global_load_lds_dwordx4, no staging registers), issued
//               from inline assembly so that the waits can be counted by hand.
//   LDS layout  an operand tile sits in LDS in the orientation it has in memory:
//                 KC  contraction index contiguous, [rows][32 k]: a lane's 8
//                     k-values are one 16-byte ds_read;
//                 RC  row index contiguous, [32 k][rows]: the lane's 8 k-values
//                     are strided and fetched with the LDS transpose read
//                     ds_read_b64_tr_b16 (two per fragment; within 16 lanes it
//                     returns to lane j, element r, element j%4 of the 8 bytes
//                     addressed by lane 4r + j/4).
//               A direct-to-LDS copy writes 1 KB per wavefront contiguously, so
//               rows cannot be padded; the 64 LDS banks are spread by an XOR
//               swizzle of the 16-byte chunk index instead, applied on the
//               global-address side of the copy and again by the readers.
//   pairings    NN (A KC, B RC)  da = g W2, dn = da W1   (weights as stored)
//               TN (A RC, B RC)  dW2 = g^T z, dW1 = da^T y, dU
//               NT (A KC, B KC)  forward  a = y W1^T, out = z W2^T
//   accumulator the MFMAs are issued with the operands exchanged (B fragment
//               first), which leaves a lane with one output row and groups of
//               four consecutive output columns.
//   two kernels lean: every tile inside the matrix, K a multiple of 32 per
//               split, the hot epilogues.  Straight-line: its epilogues issue a
//               known number of memory operations, so the copies stay counted
//               across them.  bf16 tiles leave through 4 KB of wave-private LDS
//               so that every global access covers whole 128-byte lines; fp32
//               tiles (parameter gradients, one per 256+ slices) are stored
//               from the registers, 16 bytes per lane.
//               general: any size whose contiguous dimensions are multiples of
//               8 and every epilogue; chunks outside the matrix are copied from
//               a zero-filled device array, rows/columns outside are not
//               stored, the pipeline drains after a tile's epilogue.
//   tile order  workgroup ids are dealt round-robin to the 8 XCDs (one L2
//               each): id % 8 selects a contiguous eighth of the tile list,
//               the workgroups of an XCD take consecutive tiles of it, and the
//               list walks 8 x 8 blocks of tiles, so the tiles an XCD works on
//               at one time share operand panels.
#include "hbp_common.h"
#include <atomic>
#include <type_traits>

namespace hbp {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float float2v __attribute__((ext_vector_type(2)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int BM = 256, BN = 256, BK = 32, NST = 4, NW = 8, NTHR = 64 * NW;
constexpr int A_BYTES = BM * BK * 2;            // 16 KB
constexpr int B_BYTES = BN * BK * 2;            // 16 KB
constexpr int STAGE_BYTES = A_BYTES + B_BYTES;  // 32 KB
constexpr int LDS_BYTES = NST * STAGE_BYTES;    // 128 KB
constexpr int GROUP_M = 8;                      // tile rows per block of the tile walk
constexpr int PER_SLICE = 4;                    // copies per wave per slice (2 for A, 2 for B)

__device__ uint4 g_zero_chunks[64];  // source of out-of-range chunks (zero-initialised)

// 16 bytes per lane, global -> LDS at lds_base + lane * 16.  lds_base is
// wave-uniform.  The compiler does not see this write to LDS: callers order it
// against LDS reads with a counted wait + a workgroup barrier.
__device__ __forceinline__ void dma16(const void* gptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off\n"
               :: "v"(gptr), "s"(lds_base) : "memory");
}
// the same with a wave-uniform 64-bit base and a 32-bit unsigned byte offset per lane
__device__ __forceinline__ void dma16_s(unsigned off, const void* sbase_in, unsigned lds_base) {
  // (the base is uniform by construction; say so where the register allocator has moved it to vector registers)
  const unsigned long long b = reinterpret_cast<unsigned long long>(sbase_in);
  const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)b);
  const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(b >> 32));
  const unsigned long long u = (unsigned long long)lo | ((unsigned long long)hi << 32);
  const void* sbase = reinterpret_cast<const void*>(u);
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n"
               :: "v"(off), "s"(sbase), "s"(lds_base) : "memory");
}
// at most N vector-memory operations outstanding (N <= 63), and no LDS operation
template <int N>
__device__ __forceinline__ void wait_vm_lds() {
  __builtin_amdgcn_s_waitcnt(0x0070 | (N & 15) | ((N >> 4) << 14));
}
template <int N>
__device__ __forceinline__ void wait_vm() {
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// Byte offset of this lane's chunk of copy i (of 2) relative to the first
// element of the tile's slice (the same for every slice and tile of a launch).
template <bool KC>
__device__ __forceinline__ unsigned lane_src_offset(long ld, int i, int wave, int lane) {
  const int j = wave + NW * i;
  if (KC) {
    const int r = 16 * j + (lane >> 2);
    const int c = (lane & 3) ^ ((r >> 2) & 3);
    return (unsigned)(r * ld + 8 * c) * 2u;
  } else {
    const int k = 2 * j + (lane >> 5);
    const int c = (lane & 31) ^ (4 * (k & 3));
    return (unsigned)(k * ld + 8 * c) * 2u;
  }
}
// Edge path: copies one operand tile's share of a slice (2 copies of 1 KB per
// wave) with every chunk checked against the matrix.  `base` points at the
// tile's first row (KC) or first column (RC), k0 is the slice's first
// contraction index.
template <bool KC>
__device__ __forceinline__ void issue_tile(const bf16_t* base, long ld, long rows_left, long k0, long k_end,
                                           unsigned lds_tile, int wave, int lane) {
  const bf16_t* slice = KC ? base + k0 : base + k0 * ld;   // uniform
#pragma unroll
  for (int i = 0; i < 256 / 16 / NW; ++i) {
    const int j = wave + NW * i;                // copy index within the tile: 1 KB each
    bool ok;
    const bf16_t* src;
    if (KC) {                                   // [256 rows][4 chunks]; chunk c of row r sits at c ^ (r/4 % 4)
      const int r = 16 * j + (lane >> 2);
      const int c = (lane & 3) ^ ((r >> 2) & 3);
      ok = r < rows_left && k0 + 8 * c < k_end;
      src = slice + (long)r * ld + 8 * c;
    } else {                                    // [32 k][32 chunks]; chunk c of row k sits at c ^ 4*(k % 4)
      const int k = 2 * j + (lane >> 5);
      const int c = (lane & 31) ^ (4 * (k & 3));
      ok = 8 * c < rows_left && k0 + k < k_end;
      src = slice + (long)k * ld + 8 * c;
    }
    dma16(ok ? (const void*)src : (const void*)(g_zero_chunks + lane), lds_tile + (unsigned)j * 1024u);
  }
}

// 32 rows x 16 k fragment: lane l holds row (l % 32), k = kk + 8*(l/32) .. +7
template <bool KC>
__device__ __forceinline__ bf16x8 frag(const unsigned char* tile, int row0, int kk, int lane) {
  if (KC) {
    const int r = row0 + (lane & 31);
    const int c = (kk >> 3) + (lane >> 5);
    const uint4 v = *reinterpret_cast<const uint4*>(tile + r * 64 + ((c ^ ((r >> 2) & 3)) << 4));
    return __builtin_bit_cast(bf16x8, v);
  } else {
    typedef __attribute__((address_space(3))) short4v* lds_p;
    const int s = lane & 15;
    const int e = row0 + 16 * ((lane >> 4) & 1) + 4 * (s & 3);
    const int k = kk + 8 * (lane >> 5) + (s >> 2);          // k & 3 == s >> 2 for both halves
    const int sw = 4 * (s >> 2);
    const unsigned char* p = tile + k * 512 + (((e >> 3) ^ sw) << 4) + (e & 7) * 2;
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p + 4 * 512));
    const short8v v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
  }
}

__device__ __forceinline__ float gelu_f(float a) {
  return 0.5f * a * (1.0f + erff(a * 0.70710678118654752440f));
}
__device__ __forceinline__ float gelu_grad_f(float a) {
  return 0.5f * (1.0f + erff(a * 0.70710678118654752440f)) + a * __expf(-0.5f * a * a) * 0.39894228040143267794f;
}

// 4 consecutive elements <-> 4 floats
__device__ __forceinline__ unsigned pack2(float a, float b) {   // round to nearest even (v_cvt_pk_bf16_f32)
  const float2v v = {a, b};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ void unpack4(uint2 r, float (&o)[4]) {
  o[0] = __uint_as_float(r.x << 16); o[1] = __uint_as_float(r.x & 0xFFFF0000u);
  o[2] = __uint_as_float(r.y << 16); o[3] = __uint_as_float(r.y & 0xFFFF0000u);
}
__device__ __forceinline__ void load4(const bf16_t* p, float (&o)[4]) { unpack4(*reinterpret_cast<const uint2*>(p), o); }
__device__ __forceinline__ void load4(const float* p, float (&o)[4]) {
  const float4 a = *reinterpret_cast<const float4*>(p);
  o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
}
__device__ __forceinline__ void store4(bf16_t* p, const float (&v)[4]) {
  *reinterpret_cast<uint2*>(p) = make_uint2(pack2(v[0], v[1]), pack2(v[2], v[3]));
}
__device__ __forceinline__ void store4(float* p, const float (&v)[4]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
}

// coordinates of one output tile and its share of the contraction
struct TileCoord {
  long batch, m0, n0, k_begin, k_end;
  int split, KT;
};

__device__ __forceinline__ TileCoord decode_tile(const GemmArgs& g, int t, int tiles_m, int tiles_n) {
  TileCoord c;
  const unsigned tiles_mn = (unsigned)tiles_m * tiles_n;
  const unsigned zb = (unsigned)t / tiles_mn;            // batch * split_k + split
  const unsigned rem = (unsigned)t - zb * tiles_mn;
  const unsigned grp = rem / ((unsigned)GROUP_M * tiles_n);
  const unsigned in_grp = rem - grp * GROUP_M * tiles_n;
  const unsigned left = tiles_m - grp * GROUP_M;
  const unsigned gm = left < (unsigned)GROUP_M ? left : (unsigned)GROUP_M;
  c.m0 = (long)(grp * GROUP_M + in_grp % gm) * BM;
  c.n0 = (long)(in_grp / gm) * BN;
  c.batch = zb / (unsigned)g.split_k;
  c.split = (int)(zb % (unsigned)g.split_k);
  long kchunk = (g.K + g.split_k - 1) / g.split_k;
  kchunk = (kchunk + BK - 1) / BK * BK;
  c.k_begin = (long)c.split * kchunk;
  c.k_end = c.k_begin + kchunk < g.K ? c.k_begin + kchunk : g.K;
  c.KT = c.k_end > c.k_begin ? (int)((c.k_end - c.k_begin + BK - 1) / BK) : 0;
  return c;
}

// Epilogues of the lean kernel
enum FastEpi {
  FAST_STORE = 1,      // C(bf16) = acc
  FAST_STORE_F32 = 2,  // C(fp32) = acc, also the split-K partial sums
  FAST_MUL_AUX = 3,    // C(bf16) = acc * aux
  FAST_MUL_1MZ2 = 4,   // C(bf16) = acc * (1 - aux^2)
  FAST_ADD_AUX = 5,    // C(bf16) = acc + aux
  FAST_RESID = 6,      // C(bf16) = acc + lambda[n] * aux   (forward: x_{l+1}; lambda NULL = 1)
  FAST_ACT_GELU = 7    // C(bf16) = gelu(acc), out2(bf16) = gelu'(acc)   (forward: z and act')
};

template <bool A_KC, bool B_KC, bool ACT>
__global__ __launch_bounds__(NTHR, 1) void gemm_mfma_kernel(GemmArgs g, int tiles_m, int tiles_n, long total,
                                                            long per_xcd) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2;           // phase group
  const int wm0 = grp * 128, wn0 = (wave & 3) * 64;
  const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;

  // tiles of this workgroup: t_first, t_first + t_stride, ... below t_end
  const int xcd = blockIdx.x & 7;
  const int t_stride = gridDim.x >> 3;
  const int t_first = xcd * (int)per_xcd + (blockIdx.x >> 3);
  const int t_end = (xcd + 1) * per_xcd < total ? (xcd + 1) * (int)per_xcd : (int)total;
  if (t_first >= t_end) return;

  const long lda = A_KC ? g.a_sm : g.a_sk;
  const long ldb = B_KC ? g.b_sn : g.b_sk;

  // ---- producer: the next slice of the stream to copy ----
  // All of its state is wave-uniform (scalar registers) and advanced
  // incrementally; the only per-lane values are two 32-bit source offsets.
  const bf16_t* pa = nullptr;  // producer tile's first row of A / first column of B
  const bf16_t* pb = nullptr;
  const bf16_t* qa = nullptr;  // the same, at the next slice to copy
  const bf16_t* qb = nullptr;
  const long step_a = A_KC ? BK : BK * lda;   // elements per slice
  const long step_b = B_KC ? BK : BK * ldb;
  int pt = t_first - t_stride;   // producer tile (moved onto its first tile by the first produce())
  TileCoord pc;
  int p_left = 0;             // slices of the producer tile still to copy
  long k_next = 0;            // first contraction index of the next slice
  bool p_inside = false;      // the producer tile lies fully inside the matrix
  bool p_valid = true;
  unsigned p_lds = lds0 + (unsigned)wave * 1024u;   // LDS address of this wave's first copy in the next stage
  int p_stage = 0;
  int issued = 0;             // slices issued so far
  // A wave's second copy is 128 rows (KC) or 16 k rows (RC) after its first, where the
  // swizzle repeats: same lane offset, base moved by a uniform amount.
  const unsigned offA = lane_src_offset<A_KC>(lda, 0, wave, lane);
  const unsigned offB = lane_src_offset<B_KC>(ldb, 0, wave, lane);
  const long second_a = (A_KC ? 128 : 16) * lda, second_b = (B_KC ? 128 : 16) * ldb;
  auto produce = [&]() {
    if (!p_valid) return;
    if (p_left == 0) {        // next tile with a non-empty k range
      p_valid = false;
      for (pt += t_stride; pt < t_end; pt += t_stride) {
        pc = decode_tile(g, pt, tiles_m, tiles_n);
        if (pc.KT > 0) { p_valid = true; break; }
      }
      if (!p_valid) return;
      p_left = pc.KT;
      k_next = pc.k_begin;
      p_inside = pc.m0 + BM <= g.M && pc.n0 + BN <= g.N;
      pa = reinterpret_cast<const bf16_t*>(g.A) + pc.batch * g.a_sb + (A_KC ? pc.m0 * lda : pc.m0);
      pb = reinterpret_cast<const bf16_t*>(g.B) + pc.batch * g.b_sb + (B_KC ? pc.n0 * ldb : pc.n0);
      qa = A_KC ? pa + k_next : pa + k_next * lda;
      qb = B_KC ? pb + k_next : pb + k_next * ldb;
    }
    if (p_inside && k_next + BK <= pc.k_end) {
      // interior tile, full slice: a wave-uniform base plus one 32-bit offset per lane
      dma16_s(offA, qa, p_lds);
      dma16_s(offA, qa + second_a, p_lds + NW * 1024u);
      dma16_s(offB, qb, p_lds + A_BYTES);
      dma16_s(offB, qb + second_b, p_lds + A_BYTES + NW * 1024u);
    } else {
      const unsigned st0 = p_lds - (unsigned)wave * 1024u;
      issue_tile<A_KC>(pa, lda, g.M - pc.m0, k_next, pc.k_end, st0, wave, lane);
      issue_tile<B_KC>(pb, ldb, g.N - pc.n0, k_next, pc.k_end, st0 + A_BYTES, wave, lane);
    }
    qa += step_a;
    qb += step_b;
    k_next += BK;
    --p_left;
    ++issued;
    if (++p_stage == NST) { p_stage = 0; p_lds -= (NST - 1) * STAGE_BYTES; } else p_lds += STAGE_BYTES;
  };

  // ---- consumer ----
  // acc[i][j]: lane l, element r  <->  output row wm0 + 32 i + l % 32,
  //                                    column wn0 + 32 j + 8 (r / 4) + 4 (l / 32) + r % 4
  float16v acc[4][2];
  bf16x8 fa[4][2], fb[2][2];
  auto load_frags = [&](const unsigned char* st) {
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int j = 0; j < 2; ++j) fb[j][h] = frag<B_KC>(st + A_BYTES, wn0 + 32 * j, 16 * h, lane);
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int i = 0; i < 4; ++i) fa[i][h] = frag<A_KC>(st, wm0 + 32 * i, 16 * h, lane);
  };
  auto mma_slice = [&](bool first) {
    if (first) {     // first slice of a tile: the accumulators start from zero
      const float16v zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j][0], fa[i][0], zero, 0, 0, 0);
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j][0], fa[i][0], acc[i][j], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j][1], fa[i][1], acc[i][j], 0, 0, 0);
  };

  // ---- epilogue of one tile, general form: every access guarded, every mode ----
  auto epilogue = [&](const TileCoord& tc) {
    const int rl = lane & 31, ch = (lane >> 5) * 4;
    const float* lam = g.lambda ? g.lambda + tc.batch * g.lambda_sb : nullptr;
    const bool use_aux = g.mode == EPI_MUL_AUX || g.mode == EPI_MUL_1MZ2 || g.mode == EPI_RESID ||
                         g.mode == EPI_ADD_AUX;
    const bf16_t* aux = reinterpret_cast<const bf16_t*>(g.aux) + tc.batch * g.aux_sb;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const long row = tc.m0 + wm0 + 32 * i + rl;
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const long col = tc.n0 + wn0 + 32 * j + 8 * q + ch;
          if (row >= g.M || col >= g.N) continue;
          float v[4];
#pragma unroll
          for (int x = 0; x < 4; ++x) v[x] = acc[i][j][4 * q + x];
          const long off = row * g.ldc + col;
          if (g.split_k > 1) {
            store4(reinterpret_cast<float*>(g.C) + ((long)tc.split * g.batch + tc.batch) * g.c_sb + off, v);
            continue;
          }
          if (g.addf) {
            float t[4];
            load4(g.addf + tc.batch * g.addf_sb + off, t);
#pragma unroll
            for (int x = 0; x < 4; ++x) v[x] += t[x];
          }
          float t[4] = {0.f, 0.f, 0.f, 0.f};
          if (use_aux) load4(aux + off, t);
          switch (g.mode) {
            case EPI_MUL_AUX:
#pragma unroll
              for (int x = 0; x < 4; ++x) v[x] *= t[x];
              break;
            case EPI_MUL_1MZ2:
#pragma unroll
              for (int x = 0; x < 4; ++x) v[x] *= (1.f - t[x] * t[x]);
              break;
            case EPI_ACT_GELU:
              if (ACT) {
                float d[4];
#pragma unroll
                for (int x = 0; x < 4; ++x) { d[x] = gelu_grad_f(v[x]); v[x] = gelu_f(v[x]); }
                store4(reinterpret_cast<bf16_t*>(g.out2) + tc.batch * g.out2_sb + off, d);
              }
              break;
            case EPI_ACT_TANH:
              if (ACT) {
#pragma unroll
                for (int x = 0; x < 4; ++x) v[x] = tanhf(v[x]);
              }
              break;
            case EPI_RESID:
              if (g.lambda_mn) {
                float l4[4];
                load4(reinterpret_cast<const bf16_t*>(g.lambda_mn) + tc.batch * g.aux_sb + off, l4);
#pragma unroll
                for (int x = 0; x < 4; ++x) v[x] = fmaf(l4[x], t[x], v[x]);
              } else if (lam) {
                float l4[4];
                load4(lam + col, l4);
#pragma unroll
                for (int x = 0; x < 4; ++x) v[x] = fmaf(l4[x], t[x], v[x]);
              } else {
#pragma unroll
                for (int x = 0; x < 4; ++x) v[x] += t[x];
              }
              break;
            case EPI_ADD_AUX:
#pragma unroll
              for (int x = 0; x < 4; ++x) v[x] += t[x];
              break;
            default: break;
          }
          if (g.c_is_f32)
            store4(reinterpret_cast<float*>(g.C) + tc.batch * g.c_sb + off, v);
          else
            store4(reinterpret_cast<bf16_t*>(g.C) + tc.batch * g.c_sb + off, v);
        }
    }
  };

  // ---- the stream ----
  // Barrier intervals ("ticks"): group 0 loads slice c in tick 2c and multiplies
  // it in tick 2c+1; group 1 does the same one tick later.  Slice c+3 is issued
  // in the load phase of slice c into the stage of slice c-1, which the last
  // reader (group 1, tick 2c-1) has left.  Every wave waits for its own share
  // of slice c+1 at the end of its load phase of slice c, two barriers or more
  // before the first reader of slice c+1 starts.
#pragma unroll 1
  for (int s = 0; s < NST - 1; ++s) produce();
  if (issued == 0) return;
  if (issued >= 3) wait_vm<2 * PER_SLICE>(); else if (issued == 2) wait_vm<PER_SLICE>(); else wait_vm<0>();
  __builtin_amdgcn_s_barrier();            // slice 0 is in LDS
  if (grp == 1) __builtin_amdgcn_s_barrier();   // group 1 runs one tick behind

  int ct = t_first - t_stride; // consumer tile (moved onto its first tile below)
  TileCoord cc, ec;
  cc.KT = 0;
  int ck = 0;                  // slice of the consumer tile being multiplied
  int c_stage = 0;             // its stage
  int consumed = 0;            // its index in the stream
  bool epi_pending = false;    // tile ec is complete in the accumulators
  int epi_age = 0;             // load phases whose wait still sees the last epilogue's operations
  while (true) {
    // ---------------- load phase ----------------
    if (epi_pending) {
      epilogue(ec);
      epi_age = 2;
      epi_pending = false;
    }
    if (ck == cc.KT) {         // first slice of the next tile (same walk as the producer's)
      do {
        ct += t_stride;
        cc = decode_tile(g, ct, tiles_m, tiles_n);
      } while (cc.KT == 0);
      ck = 0;
    }
    produce();                 // slice consumed + 3, into the stage of slice consumed - 1
    load_frags(smem + c_stage * STAGE_BYTES);
    const bool has_next = consumed + 1 < issued;   // the producer is always ahead while slices remain
    {
      // this wave's share of slice consumed+1 has landed once only what was issued after it is outstanding
      const int younger = has_next ? issued - consumed - 2 : 0;
      if (epi_age > 0) {        // the epilogue's stores and loads are not counted: drain
        wait_vm_lds<0>();
        --epi_age;
      } else {
        if (younger >= 2) wait_vm_lds<2 * PER_SLICE>();
        else if (younger == 1) wait_vm_lds<PER_SLICE>();
        else wait_vm_lds<0>();
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    // ---------------- compute phase ----------------
    __builtin_amdgcn_s_setprio(1);
    mma_slice(ck == 0);
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    if (++ck == cc.KT) { epi_pending = true; ec = cc; }
    if (++c_stage == NST) c_stage = 0;
    if (!has_next) break;
    ++consumed;
  }
  if (epi_pending) epilogue(ec);
  if (grp == 0) __builtin_amdgcn_s_barrier();   // matches group 1's last barrier
}


// Straight-line epilogue from the registers for a tile fully inside the matrix (fp32 output).
template <int FAST>
__device__ __forceinline__ void epilogue_fast_fn(const GemmArgs& g, const TileCoord& tc, const float16v (&acc)[4][2],
                                                 int wm0, int wn0, int lane) {
  constexpr bool HAS_AUX = FAST == FAST_MUL_AUX || FAST == FAST_MUL_1MZ2 || FAST == FAST_ADD_AUX;
  const long off0 = (tc.m0 + wm0 + (lane & 31)) * g.ldc + tc.n0 + wn0 + 4 * (lane >> 5);   // this lane's first element
  const bf16_t* aux = reinterpret_cast<const bf16_t*>(g.aux) + tc.batch * g.aux_sb + off0;
  const long cb = g.split_k > 1 ? ((long)tc.split * g.batch + tc.batch) * g.c_sb : tc.batch * g.c_sb;
  float* cf = reinterpret_cast<float*>(g.C) + cb + off0;
  bf16_t* chp = reinterpret_cast<bf16_t*>(g.C) + cb + off0;
  uint2 auxv[2][8];
  if (HAS_AUX) {
#pragma unroll
    for (int jq = 0; jq < 8; ++jq) auxv[0][jq] = *reinterpret_cast<const uint2*>(aux + 8 * jq);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (HAS_AUX && i + 1 < 4) {
#pragma unroll
      for (int jq = 0; jq < 8; ++jq)
        auxv[(i + 1) & 1][jq] = *reinterpret_cast<const uint2*>(aux + (long)(32 * (i + 1)) * g.ldc + 8 * jq);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float v[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) v[x] = acc[i][j][4 * q + x];
        if (HAS_AUX) {
          float t[4];
          unpack4(auxv[i & 1][4 * j + q], t);
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            if (FAST == FAST_MUL_AUX) v[x] *= t[x];
            else if (FAST == FAST_ADD_AUX) v[x] += t[x];
            else v[x] *= (1.f - t[x] * t[x]);
          }
        }
        const long ro = (long)(32 * i) * g.ldc + 32 * j + 8 * q;
        if (FAST == FAST_STORE_F32) store4(cf + ro, v); else store4(chp + ro, v);
      }
  }
}

// The lean form of the kernel, for launches in which every tile lies inside the
// matrix and every tile's contraction range is a multiple of 4 slices: the LDS
// stage of every step is then a compile-time constant (four steps are written
// out), the copies need two scalar pointers that advance by a constant, and a
// step is ~40 instructions next to its 16 MFMAs.  (A wavefront issues at most
// one instruction every four cycles, so the instruction count of the load phase
// is what decides whether it fits under the other group's 512 MFMA cycles.)
template <int C>
__device__ __forceinline__ void dma16_c(unsigned off, const void* sbase, unsigned lds_wave_base) {
  asm volatile("s_add_u32 m0, %2, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n"
               :: "v"(off), "s"(sbase), "s"(lds_wave_base), "n"(C) : "memory", "scc");
}

// Epilogue of a bf16 tile through 4 KB of wave-private LDS, 32 rows x 64 columns at a time: the
// accumulators (and the fused operand) change between the MFMA layout (a lane owns one row and
// groups of 4 columns) and a row layout (8 lanes cover the 128 bytes of a row), so that every
// global access of a wave covers whole 128-byte lines: 8 rows per instruction.  The 16-byte chunk
// k of row r sits at chunk k ^ (r/2 % 8) of the row (bank spread for both access shapes).
// Lanes of one wave exchange data through LDS here: the hardware executes a wave's LDS instructions in
// order, and a wave barrier between the two access shapes keeps the compiler from moving a read of one
// shape above the writes of the other (it emits no instruction).
typedef unsigned uint4v __attribute__((ext_vector_type(4)));   // (a first-class vector: stays in registers)
struct Quad16 { uint4v x0, x1, x2, x3; };   // 4 x 16 bytes per lane: 32 rows of the row layout
template <int FAST>
__device__ __forceinline__ void epilogue_staged_fn(const GemmArgs& g, const TileCoord& tc, const float16v (&acc)[4][2],
                                                   int wm0, int wn0, int lane, unsigned char* stg) {
  constexpr bool HAS_AUX = FAST == FAST_MUL_AUX || FAST == FAST_MUL_1MZ2 || FAST == FAST_ADD_AUX || FAST == FAST_RESID;
  constexpr bool TWO_OUT = FAST == FAST_ACT_GELU;
  // row layout: this lane's row within a group of 8 rows, and its chunk of the row
  const int rr = lane >> 3, rk = lane & 7;
  // MFMA layout: this lane's row within the 32, half-chunk (4 columns) within a chunk
  const int mr = lane & 31, mh = lane >> 5;
  const long off_row = (tc.m0 + wm0 + rr) * g.ldc + tc.n0 + wn0 + 8 * rk;     // row layout, first row group
  const bf16_t* aux = reinterpret_cast<const bf16_t*>(g.aux) + tc.batch * g.aux_sb + off_row;
  bf16_t* cp = reinterpret_cast<bf16_t*>(g.C) + tc.batch * g.c_sb + off_row;
  bf16_t* cp2 = TWO_OUT ? reinterpret_cast<bf16_t*>(g.out2) + tc.batch * g.out2_sb + off_row : nullptr;
  const long ld8 = 8 * g.ldc;
  // FAST_RESID: the coefficients of this lane's columns in the MFMA layout (chunk k: columns 8 k + 4 mh .. + 3)
  float lam[8][4];
  if (FAST == FAST_RESID) {
    const float* lp = g.lambda ? g.lambda + tc.batch * g.lambda_sb + tc.n0 + wn0 + 4 * mh : nullptr;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      if (lp) {
        const float4 t = *reinterpret_cast<const float4*>(lp + 8 * k);
        lam[k][0] = t.x; lam[k][1] = t.y; lam[k][2] = t.z; lam[k][3] = t.w;
      } else {
        lam[k][0] = lam[k][1] = lam[k][2] = lam[k][3] = 1.f;
      }
    }
  }
  // staging addresses, row layout: rows rr, rr + 8, rr + 16, rr + 24
  auto row_at = [&](int r) { return stg + r * 128 + ((rk ^ ((r >> 1) & 7)) << 4); };
  unsigned char* const p0 = row_at(rr);
  unsigned char* const p1 = row_at(rr + 8);
  unsigned char* const p2 = row_at(rr + 16);
  unsigned char* const p3 = row_at(rr + 24);
  unsigned char* const m_base = stg + mr * 128 + 8 * mh;
  const int m_sw = (mr >> 1) & 7;
  auto fetch = [&](Quad16& q, int round) {
    const bf16_t* a = aux + (long)(32 * round) * g.ldc;
    // (streamed once: non-temporal, so that it does not push the operand panels out of L2)
    q.x0 = __builtin_nontemporal_load(reinterpret_cast<const uint4v*>(a));
    q.x1 = __builtin_nontemporal_load(reinterpret_cast<const uint4v*>(a + ld8));
    q.x2 = __builtin_nontemporal_load(reinterpret_cast<const uint4v*>(a + 2 * ld8));
    q.x3 = __builtin_nontemporal_load(reinterpret_cast<const uint4v*>(a + 3 * ld8));
  };
  // 32 rows x 64 columns now in the staging tile (MFMA layout written): read as rows, store whole lines
  auto flush = [&](bf16_t* c) {
    __builtin_amdgcn_wave_barrier();
    const uint4v o0 = *reinterpret_cast<const uint4v*>(p0);
    const uint4v o1 = *reinterpret_cast<const uint4v*>(p1);
    const uint4v o2 = *reinterpret_cast<const uint4v*>(p2);
    const uint4v o3 = *reinterpret_cast<const uint4v*>(p3);
    __builtin_amdgcn_wave_barrier();      // the next round's writes stay behind these reads
    __builtin_nontemporal_store(o0, reinterpret_cast<uint4v*>(c));
    __builtin_nontemporal_store(o1, reinterpret_cast<uint4v*>(c + ld8));
    __builtin_nontemporal_store(o2, reinterpret_cast<uint4v*>(c + 2 * ld8));
    __builtin_nontemporal_store(o3, reinterpret_cast<uint4v*>(c + 3 * ld8));
  };
  auto round = [&](auto ic, const Quad16& q) {
    constexpr int i = decltype(ic)::value;
    uint2 auxm[8];
    uint2 second[8];        // TWO_OUT: the second output's values, packed, until the first has left the staging tile
    if (HAS_AUX) {
      *reinterpret_cast<uint4v*>(p0) = q.x0;
      *reinterpret_cast<uint4v*>(p1) = q.x1;
      *reinterpret_cast<uint4v*>(p2) = q.x2;
      *reinterpret_cast<uint4v*>(p3) = q.x3;
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int k = 0; k < 8; ++k) auxm[k] = *reinterpret_cast<const uint2*>(m_base + ((k ^ m_sw) << 4));
    }
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int qd = 0; qd < 4; ++qd) {
        float v[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) v[x] = acc[i][j][4 * qd + x];
        if (HAS_AUX) {
          float t[4];
          unpack4(auxm[4 * j + qd], t);
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            if (FAST == FAST_MUL_AUX) v[x] *= t[x];
            else if (FAST == FAST_ADD_AUX) v[x] += t[x];
            else if (FAST == FAST_RESID) v[x] = fmaf(lam[4 * j + qd][x], t[x], v[x]);
            else v[x] *= (1.f - t[x] * t[x]);
          }
        }
        if (TWO_OUT) {
          float dz[4];
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            const float a = v[x];
            const float phi = 0.5f * (1.0f + erff(a * 0.70710678118654752440f));
            v[x] = a * phi;
            dz[x] = phi + a * __expf(-0.5f * a * a) * 0.39894228040143267794f;
          }
          second[4 * j + qd] = make_uint2(pack2(dz[0], dz[1]), pack2(dz[2], dz[3]));
        }
        *reinterpret_cast<uint2*>(m_base + (((4 * j + qd) ^ m_sw) << 4)) = make_uint2(pack2(v[0], v[1]), pack2(v[2], v[3]));
      }
    flush(cp + (long)(32 * i) * g.ldc);
    if (TWO_OUT) {
#pragma unroll
      for (int k = 0; k < 8; ++k) *reinterpret_cast<uint2*>(m_base + ((k ^ m_sw) << 4)) = second[k];
      flush(cp2 + (long)(32 * i) * g.ldc);
    }
  };
  Quad16 qa = {}, qb = {};
  if (HAS_AUX) { fetch(qa, 0); fetch(qb, 1); }
  round(std::integral_constant<int, 0>(), qa);
  if (HAS_AUX) fetch(qa, 2);
  round(std::integral_constant<int, 1>(), qb);
  if (HAS_AUX) fetch(qb, 3);
  round(std::integral_constant<int, 2>(), qa);
  round(std::integral_constant<int, 3>(), qb);
}
template <int FAST> struct StagedOps {   // vector-memory operations per wave of one epilogue (a lower bound: the
  static constexpr int value = FAST == FAST_STORE_F32 ? 32 : FAST == FAST_STORE ? 16 : 32;   // waits stay safe with more)
};

constexpr int PAIR_AREA = 2 * A_BYTES;                   // 256 rows x 128 bytes: two slices of a K-contiguous operand
// Byte offset of this lane's 16 bytes of the first of a wave's four copies of a pair (rows 8 wave .. + 7 of the
// first 64; the lane's LDS place l % 8 in row l / 8 holds chunk (l % 8) ^ (row / 2 % 8) of the row's 128 bytes)
__device__ __forceinline__ unsigned pair_src_offset(long ld, int wave, int lane) {
  const int r = 8 * wave + (lane >> 3);
  const int c = (lane & 7) ^ ((r >> 1) & 7);
  return (unsigned)(r * ld + 8 * c) * 2u;
}
// 32 rows x 16 k fragment out of a pair area: lane l holds row (l % 32), chunk c0 + l / 32 of the row's eight
__device__ __forceinline__ bf16x8 frag_pair(const unsigned char* area, int row0, int c0, int lane) {
  const int r = row0 + (lane & 31);
  const int c = c0 + (lane >> 5);
  const uint4 v = *reinterpret_cast<const uint4*>(area + r * 128 + ((c ^ ((r >> 1) & 7)) << 4));
  return __builtin_bit_cast(bf16x8, v);
}

constexpr int LEAN_NST = 4;                              // 4 x 32 KB, + 4 KB per wave for the epilogue
constexpr int LEAN_LDS = LEAN_NST * STAGE_BYTES + NW * 4096;

// PAIR (A contiguous along K, every tile's range an even number of slices): A is copied two slices at a time, 128
// bytes of every row, so that each request for A takes a whole 128-byte line out of L2 (a 64-byte row segment costs
// L2 a whole line as well, and the other half is asked for again one slice later: half as much again in L2 reads
// for the pairing with one K-contiguous operand, which is bound by them).  LDS then holds two areas of 256 rows x
// 128 bytes for A (chunk k of row r at chunk k ^ (r/2 % 8)), refilled at every even step with the pair two steps
// ahead, and the ring of four 16 KB stages for B behind them; everything else is as without it.
template <bool A_KC, bool B_KC, int FAST, bool ONE_AT_A_TIME, bool PAIR>
__global__ __launch_bounds__(NTHR, 1) void gemm_mfma_lean_kernel(GemmArgs g, int tiles_m, int tiles_n, long total,
                                                                 long per_xcd) {
  static_assert(!PAIR || A_KC, "pairs of slices are copied for a K-contiguous A only");
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2;
  const int wm0 = grp * 128, wn0 = (wave & 3) * 64;
  const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
  const unsigned lds_wave = lds0 + (unsigned)wave * 1024u;

  const int xcd = blockIdx.x & 7;
  // Plain walk: every XCD takes a contiguous eighth of the tile list (small matrices: an XCD's L2 keeps a
  // matrix's panels to itself).  ONE_AT_A_TIME: blocks of (workgroups per XCD) consecutive tiles are dealt to the
  // XCDs in turn, so that at any time the whole chip works on neighbouring blocks of ONE matrix of the batch:
  // with operands too large for the caches, what the eight L2s miss is then the same panels at the same time
  // (one trip to memory instead of eight, the rest served by the memory-side cache).
  const int wpx = gridDim.x >> 3;
  const int t_stride = ONE_AT_A_TIME ? (int)gridDim.x : wpx;
  int t = (ONE_AT_A_TIME ? xcd * wpx : xcd * (int)per_xcd) + (blockIdx.x >> 3);
  const int t_end = !ONE_AT_A_TIME && (xcd + 1) * per_xcd < total ? (xcd + 1) * (int)per_xcd : (int)total;
  if (t >= t_end) return;

  const long lda = A_KC ? g.a_sm : g.a_sk;
  const long ldb = B_KC ? g.b_sn : g.b_sk;
  const long step_a = (A_KC ? BK : BK * lda) * 2, step_b = (B_KC ? BK : BK * ldb) * 2;   // bytes per slice
  // per-lane byte offsets of the wave's two copies per operand (the second is 128 rows / 16 k rows further)
  // (PAIR: copy i of 4 covers rows 64 i + 8 wave .. + 7, 8 lanes to a row; its offset is added to the scalar base)
  const unsigned offA0 = PAIR ? pair_src_offset(lda, wave, lane) : lane_src_offset<A_KC>(lda, 0, wave, lane);
  const unsigned offB0 = lane_src_offset<B_KC>(ldb, 0, wave, lane);
  const unsigned offA1 = offA0 + (unsigned)((A_KC ? 128 : 16) * lda * 2);
  const unsigned offB1 = offB0 + (unsigned)((B_KC ? 128 : 16) * ldb * 2);
  const long pair_rows64 = 64 * lda * 2;                  // bytes between the rows of consecutive copies of a pair

  // ---- producer (wave-uniform): first byte of the next slice to copy per operand, slices left in
  // the tile it copies from, that tile's index, the stage the slice goes to ----
  const unsigned char* qa;
  const unsigned char* qb;
  int p_left, pt = t;
  bool p_more = true;
  unsigned p_off = 0;      // byte offset of the producer's stage in the ring (PAIR: of its B stage behind the A areas)
  unsigned p_aoff = 0;     // PAIR: byte offset of the A area the next pair goes to
  auto aim = [&](const TileCoord& c) {
    qa = reinterpret_cast<const unsigned char*>(reinterpret_cast<const bf16_t*>(g.A) + c.batch * g.a_sb +
                                                (A_KC ? c.m0 * lda + c.k_begin : c.m0 + c.k_begin * lda));
    qb = reinterpret_cast<const unsigned char*>(reinterpret_cast<const bf16_t*>(g.B) + c.batch * g.b_sb +
                                                (B_KC ? c.n0 * ldb + c.k_begin : c.n0 + c.k_begin * ldb));
    p_left = c.KT;
  };
  auto copy_slice = [&]() {
    if (PAIR) {
      // an odd slice of its tile (an odd number of slices left): first the pair of A it completes, then its B
      if (p_left & 1) {
        const unsigned dsta = lds_wave + p_aoff;
        dma16_c<0>(offA0, qa, dsta);
        dma16_c<NW * 1024>(offA0, qa + pair_rows64, dsta);
        dma16_c<2 * NW * 1024>(offA0, qa + 2 * pair_rows64, dsta);
        dma16_c<3 * NW * 1024>(offA0, qa + 3 * pair_rows64, dsta);
        qa += 2 * step_a;
        p_aoff ^= (unsigned)PAIR_AREA;
      }
      const unsigned dst = lds_wave + 2 * PAIR_AREA + p_off;
      dma16_c<0>(offB0, qb, dst);
      dma16_c<NW * 1024>(offB1, qb, dst);
      qb += step_b;
      p_off = p_off == (LEAN_NST - 1) * B_BYTES ? 0u : p_off + B_BYTES;
    } else {
      const unsigned dst = lds_wave + p_off;
      dma16_c<0>(offA0, qa, dst);
      dma16_c<NW * 1024>(offA1, qa, dst);
      dma16_c<A_BYTES>(offB0, qb, dst);
      dma16_c<A_BYTES + NW * 1024>(offB1, qb, dst);
      qa += step_a;
      qb += step_b;
      p_off = p_off == (LEAN_NST - 1) * STAGE_BYTES ? 0u : p_off + STAGE_BYTES;
    }
    if (--p_left == 0) {
      pt += t_stride;
      if (pt < t_end) aim(decode_tile(g, pt, tiles_m, tiles_n));
      else p_more = false;
    }
  };

  float16v acc[4][2];
  bf16x8 fa[4][2], fb[2][2];
  unsigned c_off = 0;      // byte offset of the consumer's stage
  int epi_recent = 0;      // waits that still see the last epilogue's operations
  constexpr int E = StagedOps<FAST>::value;
  constexpr int AHEAD = LEAN_NST - 1;                      // slices copied ahead of the one being multiplied
  constexpr int W_PLAIN = (AHEAD - 1) * PER_SLICE;
  constexpr int W_EPI = W_PLAIN + E > 63 ? 63 : W_PLAIN + E;
  // PAIR: a wave issues 4 copies of A and 2 of B in an even step, 2 of B in an odd one.  At the end of an even
  // step c the B of slice c + 1 (issued two steps before) must have landed: what may be outstanding is what was
  // issued after it, 2 + 4 + 2 copies (and a recent epilogue's operations); at the end of an odd step the pair
  // that holds slice c + 1, issued in the step before: 2 + 2 copies.
  constexpr int W_EVEN = 8, W_EVEN_EPI = W_EVEN + E > 63 ? 63 : W_EVEN + E, W_ODD = 4;
  unsigned c_aoff = 0;     // PAIR: byte offset of the A area being read

  // One slice: load phase, barrier, compute phase, barrier.
  // Barrier intervals ("ticks"): group 0 loads slice c in tick 2c and multiplies it in tick 2c+1;
  // group 1 does the same one tick later.  Slice c+4 is issued in the load phase of slice c into
  // the stage of slice c-1, which its last reader (group 1, tick 2c-1) has left.  Every wave waits
  // for its own share of slice c+1 at the end of its load phase of slice c, a barrier or more
  // before the first reader of slice c+1 starts.
  auto step = [&](auto first_c, auto odd_c) {
    constexpr bool FIRST = decltype(first_c)::value;
    constexpr bool ODD = decltype(odd_c)::value;         // (PAIR only: the slice's place in its pair)
    const bool copying = p_more;
    if (copying) copy_slice();
    if (PAIR) {
      const unsigned char* stb = smem + 2 * PAIR_AREA + c_off;
      const unsigned char* sta = smem + c_aoff;
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int j = 0; j < 2; ++j) fb[j][h] = frag<B_KC>(stb, wn0 + 32 * j, 16 * h, lane);
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int i = 0; i < 4; ++i) fa[i][h] = frag_pair(sta, wm0 + 32 * i, (ODD ? 4 : 0) + 2 * h, lane);
      c_off = c_off == (LEAN_NST - 1) * B_BYTES ? 0u : c_off + B_BYTES;
      if (ODD) c_aoff ^= (unsigned)PAIR_AREA;
      if (!copying) wait_vm_lds<0>();
      else if (ODD) wait_vm_lds<W_ODD>();
      else if (epi_recent > 0) { wait_vm_lds<W_EVEN_EPI>(); epi_recent = 0; }
      else wait_vm_lds<W_EVEN>();
    } else {
      const unsigned char* st = smem + c_off;
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int j = 0; j < 2; ++j) fb[j][h] = frag<B_KC>(st + A_BYTES, wn0 + 32 * j, 16 * h, lane);
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int i = 0; i < 4; ++i) fa[i][h] = frag<A_KC>(st, wm0 + 32 * i, 16 * h, lane);
      c_off = c_off == (LEAN_NST - 1) * STAGE_BYTES ? 0u : c_off + STAGE_BYTES;
      // this wave's share of the next slice has landed once only what it issued for the slices after
      // that one (and a recent epilogue's operations, which lie among them) is outstanding
      if (!copying) wait_vm_lds<0>();
      else if (epi_recent > 0) { wait_vm_lds<W_EPI>(); --epi_recent; }
      else wait_vm_lds<W_PLAIN>();
    }
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(1);
    const float16v zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j][0], fa[i][0], FIRST ? zero : acc[i][j], 0, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j][1], fa[i][1], acc[i][j], 0, 0, 0);
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
  };

  TileCoord cc = decode_tile(g, t, tiles_m, tiles_n);
  aim(cc);
  int pro = 0;             // slices copied before the first step
#pragma unroll 1
  for (; pro < AHEAD && p_more; ++pro) copy_slice();
  // slice 0 has landed once at most the pro - 1 slices after it are outstanding
  if (PAIR) {              // (issued: B of slice 0, the first pair of A, B of slices 1 and 2)
    if (pro == 3) wait_vm<4>(); else wait_vm<0>();
  } else if (pro >= 4) wait_vm<3 * PER_SLICE>(); else if (pro == 3) wait_vm<2 * PER_SLICE>();
  else if (pro == 2) wait_vm<PER_SLICE>(); else wait_vm<0>();
  __builtin_amdgcn_s_barrier();                 // slice 0 is in LDS
  if (grp == 1) __builtin_amdgcn_s_barrier();   // group 1 runs one tick behind

  while (true) {
    if (PAIR) {
      step(std::true_type(), std::false_type());
      step(std::false_type(), std::true_type());
#pragma unroll 1
      for (int k = 2; k < cc.KT; k += 2) {
        step(std::false_type(), std::false_type());
        step(std::false_type(), std::true_type());
      }
    } else {
      step(std::true_type(), std::false_type());
#pragma unroll 1
      for (int k = 1; k < cc.KT; ++k) step(std::false_type(), std::false_type());
    }
    if (FAST == FAST_STORE_F32) epilogue_fast_fn<FAST>(g, cc, acc, wm0, wn0, lane);
    else epilogue_staged_fn<FAST>(g, cc, acc, wm0, wn0, lane, smem + LEAN_NST * STAGE_BYTES + wave * 4096);
    epi_recent = AHEAD - 1;
    t += t_stride;
    if (t >= t_end) break;
    cc = decode_tile(g, t, tiles_m, tiles_n);
  }
  if (grp == 0) __builtin_amdgcn_s_barrier();   // matches group 1's last barrier
}

// Raises a kernel's dynamic shared-memory limit once per device (one flag array per kernel instantiation; setting
// the attribute twice from two threads is harmless, so a relaxed flag is enough).
constexpr int MAX_DEVICES = 64;
inline hipError_t raise_lds_limit(const void* kern, int bytes, std::atomic<bool> (&done)[MAX_DEVICES]) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  if (done[dev].load(std::memory_order_acquire)) return hipSuccess;
  e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e != hipSuccess) return e;
  done[dev].store(true, std::memory_order_release);
  return hipSuccess;
}

template <bool A_KC, bool B_KC, int FAST, bool ONE_AT_A_TIME, bool PAIR>
hipError_t launch_lean_walk(const GemmArgs& g, hipStream_t s) {
  static std::atomic<bool> attr_set[MAX_DEVICES];
  auto kern = gemm_mfma_lean_kernel<A_KC, B_KC, FAST, ONE_AT_A_TIME, PAIR>;
  {
    hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(kern), LEAN_LDS, attr_set);
    if (e != hipSuccess) return e;
  }
  const int tiles_m = (int)(g.M / BM), tiles_n = (int)(g.N / BN);
  const long total = (long)tiles_m * tiles_n * g.batch * g.split_k;
  const long per_xcd = (total + 7) / 8;
  const long wg_per_xcd = per_xcd < 32 ? per_xcd : 32;
  const int lds = LEAN_LDS;
  hipLaunchKernelGGL(kern, dim3((unsigned)(wg_per_xcd * 8)), dim3(NTHR), lds, s, g, tiles_m, tiles_n, total, per_xcd);
  return hipGetLastError();
}
template <bool A_KC, bool B_KC, int FAST>
hipError_t launch_lean(const GemmArgs& g, hipStream_t s) {
  // a batch of matrices whose operands run to tens of megabytes each: the chip takes them one at a time (measured
  // on 96 blocks of 16384 x 8192 x 2048: 8-10 % faster; on 32 blocks of 8192 x 2048 x 512: 10 % slower)
  const bool one_at_a_time = g.batch > 1 && (g.M + g.N) * g.K * 2 >= (64L << 20);
  if constexpr (A_KC) {
    // Every tile's share of K an even number of slices: A in pairs of slices.  Measured: 2-10 % on matrices that
    // the caches hold (L2 reads down by a third); on the one-at-a-time walk over 96 blocks of 16384 x 8192 x 2048
    // the same time (fewer cycles at a lower clock: the chip is at its power limit there) with twice the fills from
    // memory, the pairs being asked for closer to their use: not taken there.
    if (!one_at_a_time && g.K % ((long)g.split_k * 2 * BK) == 0)
      return launch_lean_walk<A_KC, B_KC, FAST, false, true>(g, s);
  }
  return one_at_a_time ? launch_lean_walk<A_KC, B_KC, FAST, true, false>(g, s)
                       : launch_lean_walk<A_KC, B_KC, FAST, false, false>(g, s);
}
// every tile inside the matrix, every tile's share of K a whole number of slices
inline bool lean_ok(const GemmArgs& g) {
  return g.M % BM == 0 && g.N % BN == 0 && g.K % ((long)g.split_k * BK) == 0;
}

template <bool A_KC, bool B_KC, bool ACT>
hipError_t launch_variant(const GemmArgs& g, hipStream_t s) {
  static std::atomic<bool> attr_set[MAX_DEVICES];
  auto kern = gemm_mfma_kernel<A_KC, B_KC, ACT>;
  {
    hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(kern), LDS_BYTES + 8192, attr_set);
    if (e != hipSuccess) return e;
  }
  const int tiles_m = (int)((g.M + BM - 1) / BM), tiles_n = (int)((g.N + BN - 1) / BN);
  const long total = (long)tiles_m * tiles_n * g.batch * g.split_k;
  const long per_xcd = (total + 7) / 8;
  const long wg_per_xcd = per_xcd < 32 ? per_xcd : 32;   // 32 CUs per XCD, one workgroup each
  hipLaunchKernelGGL(kern, dim3((unsigned)(wg_per_xcd * 8)), dim3(NTHR), LDS_BYTES, s, g, tiles_m, tiles_n, total,
                     per_xcd);
  return hipGetLastError();
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

bool launch_gemm_mfma(const GemmArgs& g, hipStream_t s, hipError_t* err) {
  *err = hipSuccess;
  const bool a_kc = g.a_sk == 1, a_rc = g.a_sm == 1;
  const bool b_kc = g.b_sk == 1, b_rc = g.b_sn == 1;
  if (!(a_kc || a_rc) || !(b_kc || b_rc)) return false;
  const long lda = a_kc ? g.a_sm : g.a_sk, ldb = b_kc ? g.b_sn : g.b_sk;
  // 16-byte accesses everywhere: contiguous extents, leading dimensions and batch strides in multiples of 8
  if ((a_kc ? g.K : g.M) % 8 || (b_kc ? g.K : g.N) % 8 || g.N % 8) return false;
  if (lda % 8 || ldb % 8 || g.ldc % 8 || g.a_sb % 8 || g.b_sb % 8 || g.c_sb % 8) return false;
  if (g.aux_sb % 8 || g.out2_sb % 8 || g.addf_sb % 8 || g.lambda_sb % 8) return false;
  if (!aligned16(g.A) || !aligned16(g.B) || !aligned16(g.C) || !aligned16(g.aux) || !aligned16(g.out2) ||
      !aligned16(g.addf) || !aligned16(g.lambda) || !aligned16(g.lambda_mn))
    return false;
  if (lda > (1L << 22) || ldb > (1L << 22)) return false;   // per-lane source offsets are 32-bit
  if (g.split_k > 1 && g.mode != EPI_STORE) return false;
  if (g.M <= 0 || g.N <= 0 || g.K <= 0 || g.batch <= 0 || g.split_k <= 0) return false;
  const bool act = g.mode == EPI_ACT_GELU || g.mode == EPI_ACT_TANH;
  const bool plain = g.mode == EPI_STORE && !g.addf;
  const bool lean = lean_ok(g);
  const bool bf16_out = !g.addf && !g.c_is_f32 && g.split_k == 1;
  if (a_kc && b_rc && !act) {            // VJP contractions
    // Row or column counts that are no multiple of the tile (any number of tokens, any width): the whole tiles go
    // to the aligned kernel, the remaining columns and then the remaining rows to the general one in launches of
    // their own.  The parts write disjoint blocks of C.
    const bool fast_mode = g.mode == EPI_STORE || g.mode == EPI_MUL_AUX || g.mode == EPI_MUL_1MZ2 || g.mode == EPI_ADD_AUX;
    if (!lean && bf16_out && fast_mode && g.K % BK == 0) {
      if (g.N > BN && g.N % BN != 0) {
        GemmArgs head = g, tail = g;
        head.N = g.N / BN * BN;
        tail.N = g.N - head.N;
        tail.B = reinterpret_cast<const bf16_t*>(g.B) + head.N;
        tail.C = reinterpret_cast<bf16_t*>(g.C) + head.N;
        if (g.aux) tail.aux = reinterpret_cast<const bf16_t*>(g.aux) + head.N;
        hipError_t e1 = hipSuccess;
        if (!launch_gemm_mfma(head, s, &e1)) { *err = launch_variant<true, false, false>(g, s); return true; }
        if (e1 != hipSuccess) { *err = e1; return true; }
        *err = launch_variant<true, false, false>(tail, s);
        return true;
      }
      if (g.M > BM && g.M % BM != 0 && g.N % BN == 0) {
        GemmArgs head = g, tail = g;
        head.M = g.M / BM * BM;
        tail.M = g.M - head.M;
        tail.A = reinterpret_cast<const bf16_t*>(g.A) + head.M * g.a_sm;
        tail.C = reinterpret_cast<bf16_t*>(g.C) + head.M * g.ldc;
        if (g.aux) tail.aux = reinterpret_cast<const bf16_t*>(g.aux) + head.M * g.ldc;
        hipError_t e1 = hipSuccess;
        if (!launch_gemm_mfma(head, s, &e1)) { *err = launch_variant<true, false, false>(g, s); return true; }
        if (e1 != hipSuccess) { *err = e1; return true; }
        *err = launch_variant<true, false, false>(tail, s);
        return true;
      }
    }
    if (lean && bf16_out && g.mode == EPI_STORE) *err = launch_lean<true, false, FAST_STORE>(g, s);
    else if (lean && bf16_out && g.mode == EPI_MUL_AUX) *err = launch_lean<true, false, FAST_MUL_AUX>(g, s);
    else if (lean && bf16_out && g.mode == EPI_MUL_1MZ2) *err = launch_lean<true, false, FAST_MUL_1MZ2>(g, s);
    else if (lean && bf16_out && g.mode == EPI_ADD_AUX) *err = launch_lean<true, false, FAST_ADD_AUX>(g, s);
    else *err = launch_variant<true, false, false>(g, s);
  } else if (a_rc && b_rc && !act) {     // parameter gradients
    // the same split for widths that are no multiple of the tile (fp32 result or split-K partial sums)
    if (!lean && plain && (g.c_is_f32 || g.split_k > 1) && g.K % ((long)g.split_k * BK) == 0) {
      const bool by_rows = g.M > BM && g.M % BM != 0;
      const bool by_cols = !by_rows && g.N > BN && g.N % BN != 0 && g.M % BM == 0;
      if (by_rows || by_cols) {
        GemmArgs head = g, tail = g;
        if (by_rows) {
          head.M = g.M / BM * BM;
          tail.M = g.M - head.M;
          tail.A = reinterpret_cast<const bf16_t*>(g.A) + head.M;          // a_sm == 1
          tail.C = reinterpret_cast<float*>(g.C) + head.M * g.ldc;
        } else {
          head.N = g.N / BN * BN;
          tail.N = g.N - head.N;
          tail.B = reinterpret_cast<const bf16_t*>(g.B) + head.N;          // b_sn == 1
          tail.C = reinterpret_cast<float*>(g.C) + head.N;
        }
        hipError_t e1 = hipSuccess;
        if (!launch_gemm_mfma(head, s, &e1)) { *err = launch_variant<false, false, false>(g, s); return true; }
        if (e1 != hipSuccess) { *err = e1; return true; }
        *err = launch_variant<false, false, false>(tail, s);
        return true;
      }
    }
    if (lean && plain && (g.c_is_f32 || g.split_k > 1)) *err = launch_lean<false, false, FAST_STORE_F32>(g, s);
    else *err = launch_variant<false, false, false>(g, s);
  } else if (a_kc && b_kc) {             // forward; VJP contractions against transposed weights
    if (lean && bf16_out && g.mode == EPI_ACT_GELU && g.out2) *err = launch_lean<true, true, FAST_ACT_GELU>(g, s);
    else if (lean && bf16_out && g.mode == EPI_RESID && g.aux && !g.lambda_mn) *err = launch_lean<true, true, FAST_RESID>(g, s);
    else if (lean && bf16_out && g.mode == EPI_STORE) *err = launch_lean<true, true, FAST_STORE>(g, s);
    else if (lean && bf16_out && g.mode == EPI_MUL_AUX) *err = launch_lean<true, true, FAST_MUL_AUX>(g, s);
    else if (lean && bf16_out && g.mode == EPI_MUL_1MZ2) *err = launch_lean<true, true, FAST_MUL_1MZ2>(g, s);
    else if (lean && bf16_out && g.mode == EPI_ADD_AUX) *err = launch_lean<true, true, FAST_ADD_AUX>(g, s);
    else *err = act ? launch_variant<true, true, true>(g, s) : launch_variant<true, true, false>(g, s);
  } else {
    return false;
  }
  return true;
}

}  // namespace hbp
