// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32
// accumulate) for the VJP and parameter-gradient contractions.
//
// Shape of the kernel
//   workgroup   8 wavefronts (2 x 4), output tile 256 x 256, one workgroup per
//               CU; a wavefront owns 128 x 64 = 4 x 2 MFMA blocks of 32 x 32 (128
//               accumulator registers per lane).  The 256 x 256 tile is what
//               keeps the L2 -> LDS stream (the measured limiter, ~14 TB/s over
//               the chip) below the MFMA rate: 128 flop per byte copied.
//   persistent  one workgroup per CU walks a list of tiles.  The K slices of all
//               its tiles form one stream through a ring of 4 LDS stages, so the
//               first slices of the next tile are already in flight while the
//               current tile's epilogue runs: no per-tile fill latency.
//   K pipeline  slices of 32 (32 KB per stage); a slice is copied global -> LDS
//               directly (global_load_lds_dwordx4, no staging registers) up to
//               three slices ahead of the one being multiplied; one barrier per
//               slice.  Fragments of the next MFMA group are read from LDS
//               while the current group's MFMAs run.
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
//   edges       chunks outside the matrix are copied from a zero-filled device
//               array, rows/columns outside are not stored: any size whose
//               contiguous dimensions are multiples of 8 is covered.
//   epilogue    accumulators pass through 4 KB of wave-private LDS (16 rows at a
//               time, XOR-swizzled) so that every global access (output and the
//               fused element-wise operand) is a 16-byte row-contiguous access.
//   tile order  workgroup ids are dealt round-robin to the 8 XCDs (one L2
//               each): id % 8 selects a contiguous eighth of the tile list,
//               the workgroups of an XCD take consecutive tiles of it, and the
//               list walks 8 x 8 blocks of tiles, so the tiles an XCD works on
//               at one time share operand panels.
#include "hbp_common.h"

namespace hbp {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int BM = 256, BN = 256, BK = 32, NST = 4, NW = 8, NTHR = 64 * NW;
constexpr int A_BYTES = BM * BK * 2;            // 16 KB
constexpr int B_BYTES = BN * BK * 2;            // 16 KB
constexpr int STAGE_BYTES = A_BYTES + B_BYTES;  // 32 KB
constexpr int RING_BYTES = NST * STAGE_BYTES;   // 128 KB
constexpr int EPI_WAVE_BYTES = 16 * 64 * 4;     // 16 rows x 64 fp32 per wave
constexpr int LDS_BYTES = RING_BYTES + NW * EPI_WAVE_BYTES;  // 160 KB: the whole CU
constexpr int GROUP_M = 8;                      // tile rows per block of the tile walk
constexpr int PER_SLICE = 4;                    // copies per wave per slice (2 for A, 2 for B)

__device__ uint4 g_zero_chunks[64];  // source of out-of-range chunks (zero-initialised)

// 16 bytes per lane, global -> LDS at lds_base + lane * 16.  lds_base is
// wave-uniform.  The compiler does not see this write to LDS: callers order it
// against LDS reads with wait_vm() + __syncthreads().
__device__ __forceinline__ void dma16(const void* gptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off\n"
               :: "v"(gptr), "s"(lds_base) : "memory");
}
// the same with a wave-uniform 64-bit base and a 32-bit unsigned byte offset per lane
__device__ __forceinline__ void dma16_s(unsigned off, const void* sbase, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n"
               :: "v"(off), "s"(sbase), "s"(lds_base) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vm() {   // at most N vector-memory operations outstanding
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}
// at most n slices' worth of this wave's copies outstanding
__device__ __forceinline__ void wait_slices(int n) {
  if (n >= 2) wait_vm<2 * PER_SLICE>();
  else if (n == 1) wait_vm<PER_SLICE>();
  else wait_vm<0>();
}

// Hides a value's origin from the optimiser: addresses derived from a laundered
// lane id are rebuilt where they are used instead of being hoisted out of the
// persistent loop and kept (or spilled) across the MFMA blocks.
__device__ __forceinline__ int launder(int v) {
  asm volatile("" : "+v"(v));
  return v;
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
                                           unsigned lds_tile, int wave, int lane_in) {
  const int lane = launder(lane_in);
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

// Epilogue specialisations.  For tiles that lie fully inside the matrix the hot
// epilogues are straight-line code: the number of vector-memory operations they
// issue is then a constant, which (a) lets the compiler wait for the fused
// operand with an exact count instead of draining the stores before it, and
// (b) lets the K pipeline count its copies across the epilogue.  Everything
// else (edge tiles, forward-pass epilogues) takes the general, guarded path.
enum FastEpi {
  FAST_NONE = 0,       // general path only (ACT: with the activation epilogues)
  FAST_STORE = 1,      // C(bf16) = acc
  FAST_STORE_F32 = 2,  // C(fp32) = acc, also the split-K partial sums
  FAST_MUL_AUX = 3,    // C(bf16) = acc * aux
  FAST_MUL_1MZ2 = 4,   // C(bf16) = acc * (1 - aux^2)
  FAST_ADD_AUX = 5     // C(bf16) = acc + aux
};
template <int FAST> struct FastOps {   // vector-memory operations per wave of one fast epilogue
  static constexpr int value = FAST == FAST_STORE ? 16 : FAST == FAST_STORE_F32 ? 32 : FAST == FAST_NONE ? 0 : 32;
};

template <bool A_KC, bool B_KC, bool ACT, int FAST>
__global__ __launch_bounds__(NTHR, 1) void gemm_mfma_kernel(GemmArgs g, int tiles_m, int tiles_n, long total,
                                                            long per_xcd) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave >> 2) * 128, wn0 = (wave & 3) * 64;
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
  // incrementally; the only per-lane values are four 32-bit source offsets.
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
  float16v acc[4][2];
  auto zero_acc = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  };
  // A slice is consumed in four groups of 2 x 2 MFMA blocks (k half, row half).
  // The A fragments of group g+1 are read from LDS while the MFMAs of group g
  // run, and the first fragments of the next slice while the last group runs.
  auto load_b = [&](const unsigned char* bt, int h, bf16x8 (&b)[2], int ln) {   // k half h of the slice
#pragma unroll
    for (int j = 0; j < 2; ++j) b[j] = frag<B_KC>(bt, wn0 + 32 * j, 16 * h, ln);
  };
  auto load_a = [&](const unsigned char* at, int grp, bf16x8 (&a)[2], int ln) {
#pragma unroll
    for (int ii = 0; ii < 2; ++ii) a[ii] = frag<A_KC>(at, wm0 + 32 * ((grp & 1) * 2 + ii), 16 * (grp >> 1), ln);
  };
  auto mma = [&](int grp, const bf16x8 (&a)[2], const bf16x8 (&b)[2][2]) {
#pragma unroll
    for (int ii = 0; ii < 2; ++ii)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int i = (grp & 1) * 2 + ii;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ii], b[grp >> 1][j], acc[i][j], 0, 0, 0);
      }
  };

  // ---- epilogue of one tile (wave-private; no workgroup barrier inside) ----
  float* stage = reinterpret_cast<float*>(smem + RING_BYTES + wave * EPI_WAVE_BYTES);
  auto epilogue = [&](const TileCoord& tc) {
    // (addresses are rebuilt from the lane id per tile; see launder())
    const int le = launder(lane);
    const int er = le >> 3;         // row within a group of 8
    const int ec = (le & 7) * 8;    // first of 8 columns
    const long col = tc.n0 + wn0 + ec;
    const bool col_ok = col < g.N;
    const float* lam = g.lambda ? g.lambda + tc.batch * g.lambda_sb : nullptr;
    const bool use_aux = g.split_k == 1 && (g.mode == EPI_MUL_AUX || g.mode == EPI_MUL_1MZ2 ||
                                            g.mode == EPI_RESID || g.mode == EPI_ADD_AUX);
    const bf16_t* aux = reinterpret_cast<const bf16_t*>(g.aux) + tc.batch * g.aux_sb;
    uint4 auxv[2][4];
    auto fetch_aux = [&](int i, uint4 (&dst)[4]) {   // the fused operand of 32 rows: 4 x 16 bytes per lane
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const long row = tc.m0 + wm0 + 32 * i + er + 8 * q;
        if (use_aux && row < g.M && col_ok)
          dst[q] = *reinterpret_cast<const uint4*>(aux + row * g.ldc + col);
        else
          dst[q] = make_uint4(0u, 0u, 0u, 0u);
      }
    };
    fetch_aux(0, auxv[0]);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (i + 1 < 4) fetch_aux(i + 1, auxv[(i + 1) & 1]);
#pragma unroll
      for (int h = 0; h < 2; ++h) {             // rows 16h .. 16h+15 of the 32: accumulator elements 8h .. 8h+7
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int rr = 0; rr < 8; ++rr) {
            const int r = 8 * h + rr;
            const int lr = ((r >> 2) & 1) * 8 + (lane >> 5) * 4 + (r & 3);
            const int c = j * 32 + (lane & 31);
            const int sw = (lr & 1) | (((lr >> 2) & 1) << 3);
            stage[lr * 64 + ((((c >> 2) ^ sw) << 2) | (c & 3))] = acc[i][j][r];
          }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int q2 = 0; q2 < 2; ++q2) {
          const int lr = er + 8 * q2;
          const int sw = (lr & 1) | (((lr >> 2) & 1) << 3);
          const long row = tc.m0 + wm0 + 32 * i + 16 * h + lr;
          float v[8];
          {
            const float4 lo = *reinterpret_cast<const float4*>(stage + lr * 64 + ((((ec >> 2)) ^ sw) << 2));
            const float4 hi = *reinterpret_cast<const float4*>(stage + lr * 64 + ((((ec >> 2) + 1) ^ sw) << 2));
            v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w;
            v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
          }
          if (row >= g.M || !col_ok) continue;
          const long off = row * g.ldc + col;
          if (g.split_k > 1) {
            float* P = reinterpret_cast<float*>(g.C) + ((long)tc.split * g.batch + tc.batch) * g.c_sb + off;
            store8(P, v);
            continue;
          }
          if (g.addf) {
            float t8[8];
            load8(g.addf + tc.batch * g.addf_sb + off, t8);
#pragma unroll
            for (int x = 0; x < 8; ++x) v[x] += t8[x];
          }
          float t8[8];
          {
            const uint4 a4 = auxv[i & 1][2 * h + q2];
            const unsigned int w4[4] = {a4.x, a4.y, a4.z, a4.w};
#pragma unroll
            for (int x = 0; x < 4; ++x) {
              t8[2 * x] = __uint_as_float(w4[x] << 16);
              t8[2 * x + 1] = __uint_as_float(w4[x] & 0xFFFF0000u);
            }
          }
          switch (g.mode) {
            case EPI_MUL_AUX:
#pragma unroll
              for (int x = 0; x < 8; ++x) v[x] *= t8[x];
              break;
            case EPI_MUL_1MZ2:
#pragma unroll
              for (int x = 0; x < 8; ++x) v[x] *= (1.f - t8[x] * t8[x]);
              break;
            case EPI_ACT_GELU: if (ACT) {
              float d8[8];
#pragma unroll
              for (int x = 0; x < 8; ++x) { d8[x] = gelu_grad_f(v[x]); v[x] = gelu_f(v[x]); }
              store8(reinterpret_cast<bf16_t*>(g.out2) + tc.batch * g.out2_sb + off, d8);
              break;
            }
            case EPI_ACT_TANH:
              if (ACT) {
#pragma unroll
                for (int x = 0; x < 8; ++x) v[x] = tanhf(v[x]);
              }
              break;
            case EPI_RESID:
              if (lam) {
                float l8[8];
                load8(lam + col, l8);
#pragma unroll
                for (int x = 0; x < 8; ++x) v[x] = fmaf(l8[x], t8[x], v[x]);
              } else {
#pragma unroll
                for (int x = 0; x < 8; ++x) v[x] += t8[x];
              }
              break;
            case EPI_ADD_AUX:
#pragma unroll
              for (int x = 0; x < 8; ++x) v[x] += t8[x];
              break;
            default: break;
          }
          if (g.c_is_f32)
            store8(reinterpret_cast<float*>(g.C) + tc.batch * g.c_sb + off, v);
          else
            store8(reinterpret_cast<bf16_t*>(g.C) + tc.batch * g.c_sb + off, v);
        }
        __builtin_amdgcn_wave_barrier();
      }
    }
  };

  // Straight-line epilogue for a tile fully inside the matrix (FAST != 0).
  auto epilogue_fast = [&](const TileCoord& tc) {
    const int le = launder(lane);
    const int er = le >> 3;
    const int ec = (le & 7) * 8;
    constexpr bool HAS_AUX = FAST == FAST_MUL_AUX || FAST == FAST_MUL_1MZ2 || FAST == FAST_ADD_AUX;
    const long off0 = (tc.m0 + wm0 + er) * g.ldc + tc.n0 + wn0 + ec;   // this lane's first element
    const bf16_t* aux = reinterpret_cast<const bf16_t*>(g.aux) + tc.batch * g.aux_sb + off0;
    const long cb = g.split_k > 1 ? ((long)tc.split * g.batch + tc.batch) * g.c_sb : tc.batch * g.c_sb;
    float* cf = reinterpret_cast<float*>(g.C) + cb + off0;
    bf16_t* ch = reinterpret_cast<bf16_t*>(g.C) + cb + off0;
    uint4 auxv[2][4];
    if (HAS_AUX) {
#pragma unroll
      for (int q = 0; q < 4; ++q) auxv[0][q] = *reinterpret_cast<const uint4*>(aux + (long)(8 * q) * g.ldc);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (HAS_AUX && i + 1 < 4) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
          auxv[(i + 1) & 1][q] = *reinterpret_cast<const uint4*>(aux + (long)(32 * (i + 1) + 8 * q) * g.ldc);
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int rr = 0; rr < 8; ++rr) {
            const int r = 8 * h + rr;
            const int lr = ((r >> 2) & 1) * 8 + (lane >> 5) * 4 + (r & 3);
            const int c = j * 32 + (lane & 31);
            const int sw = (lr & 1) | (((lr >> 2) & 1) << 3);
            stage[lr * 64 + ((((c >> 2) ^ sw) << 2) | (c & 3))] = acc[i][j][r];
          }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int q2 = 0; q2 < 2; ++q2) {
          const int lr = er + 8 * q2;
          const int sw = (lr & 1) | (((lr >> 2) & 1) << 3);
          float v[8];
          {
            const float4 lo = *reinterpret_cast<const float4*>(stage + lr * 64 + ((((ec >> 2)) ^ sw) << 2));
            const float4 hi = *reinterpret_cast<const float4*>(stage + lr * 64 + ((((ec >> 2) + 1) ^ sw) << 2));
            v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w;
            v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
          }
          if (HAS_AUX) {
            const uint4 a4 = auxv[i & 1][2 * h + q2];
            const unsigned int w4[4] = {a4.x, a4.y, a4.z, a4.w};
#pragma unroll
            for (int x = 0; x < 4; ++x) {
              const float t0 = __uint_as_float(w4[x] << 16), t1 = __uint_as_float(w4[x] & 0xFFFF0000u);
              if (FAST == FAST_MUL_AUX) { v[2 * x] *= t0; v[2 * x + 1] *= t1; }
              else if (FAST == FAST_ADD_AUX) { v[2 * x] += t0; v[2 * x + 1] += t1; }
              else { v[2 * x] *= (1.f - t0 * t0); v[2 * x + 1] *= (1.f - t1 * t1); }
            }
          }
          const long ro = (long)(32 * i + 16 * h + 8 * q2) * g.ldc;
          if (FAST == FAST_STORE_F32) store8(cf + ro, v); else store8(ch + ro, v);
        }
        __builtin_amdgcn_wave_barrier();
      }
    }
  };

  // ---- the stream ----
  // Ring use while slice c is multiplied: stage c%4 is read, slice c+1 has
  // landed (or is landing), slice c+2 is in flight, and the stage of slice c-1
  // is refilled with slice c+3.  The hand-over to slice c+1 (wait for its
  // copies, barrier, issue the next copy) sits in the middle of slice c's MFMAs,
  // whose operands are already in registers, so the matrix cores have work
  // while the waves meet at the barrier.
#pragma unroll 1
  for (int s = 0; s < NST - 1; ++s) produce();
  if (issued == 0) return;

  bf16x8 bcur[2][2], a0[2], a1[2];
  wait_slices(issued - 1);     // slice 0 has landed (this wave's part)
  __syncthreads();             // ... and every other wave's
  load_b(smem + A_BYTES, 0, bcur[0], lane);
  load_a(smem, 0, a0, lane);

  int ct = t_first - t_stride; // consumer tile (moved onto its first tile below)
  TileCoord cc;
  cc.KT = 0;
  int ck = 0;                  // slice of the consumer tile being multiplied
  int c_stage = 0;             // its stage
  int consumed = 0;            // its index in the stream
  int epi_ops = -1;            // >= 0: an epilogue issued that many operations after the copies in flight;
                               // -2, -1: none pending (two hand-overs after an epilogue still see its operations)
  int epi_age = 0;
  while (true) {
    if (ck == cc.KT) {         // first slice of the next tile (same walk as the producer's)
      do {
        ct += t_stride;
        cc = decode_tile(g, ct, tiles_m, tiles_n);
      } while (cc.KT == 0);
      ck = 0;
      zero_acc();
    }
    // The fragment addresses are rebuilt from the lane id in every slice rather
    // than kept in registers across the loop (the accumulators need the space).
    const int ln = lane;
    const unsigned char* at = smem + c_stage * STAGE_BYTES;
    load_b(at + A_BYTES, 1, bcur[1], ln);
    load_a(at, 1, a1, ln);
    mma(0, a0, bcur);
    __builtin_amdgcn_sched_barrier(0);
    load_a(at, 2, a0, ln);
    mma(1, a1, bcur);
    __builtin_amdgcn_sched_barrier(0);
    const bool has_next = consumed + 1 < issued;   // the producer is always ahead while slices remain
    if (has_next) {
      // slice consumed+1 has landed once only the slices issued after it are outstanding
      // (for two hand-overs after an epilogue its operations are younger than the
      // copies waited for: they are counted if their number is known, else drained)
      const int younger = issued - consumed - 2;
      if (epi_age > 0) {
        if (epi_ops < 0) wait_vm<0>();
        else if (younger >= 1) wait_vm<PER_SLICE + FastOps<FAST>::value>();
        else wait_vm<FastOps<FAST>::value>();
        --epi_age;
      } else {
        wait_slices(younger);
      }
      __syncthreads();   // every wave's part of it is in LDS; everyone is done reading slice consumed-1
      produce();         // into the stage of slice consumed-1
    }
    __builtin_amdgcn_sched_barrier(0);
    const bool tile_done = ++ck == cc.KT;
    if (++c_stage == NST) c_stage = 0;
    const unsigned char* an = smem + c_stage * STAGE_BYTES;
    const bool ahead = has_next && !tile_done;   // first fragments of the next slice under the last MFMAs
    load_a(at, 3, a1, ln);
    if (ahead) load_b(an + A_BYTES, 0, bcur[0], ln);
    mma(2, a0, bcur);
    __builtin_amdgcn_sched_barrier(0);
    if (ahead) load_a(an, 0, a0, ln);
    mma(3, a1, bcur);
    __builtin_amdgcn_sched_barrier(0);
    if (tile_done) {
      if (FAST != FAST_NONE && cc.m0 + BM <= g.M && cc.n0 + BN <= g.N) {
        epilogue_fast(cc);
        epi_ops = FastOps<FAST>::value;
      } else {
        epilogue(cc);
        epi_ops = -1;
      }
      epi_age = 2;
      if (has_next) {
        load_b(an + A_BYTES, 0, bcur[0], ln);
        load_a(an, 0, a0, ln);
      }
    }
    if (!has_next) break;
    ++consumed;
  }
}

template <bool A_KC, bool B_KC, bool ACT, int FAST>
hipError_t launch_variant(const GemmArgs& g, hipStream_t s) {
  static bool attr_set = false;
  auto kern = gemm_mfma_kernel<A_KC, B_KC, ACT, FAST>;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
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
      !aligned16(g.addf) || !aligned16(g.lambda))
    return false;
  if (g.split_k > 1 && g.mode != EPI_STORE) return false;
  if (g.M <= 0 || g.N <= 0 || g.K <= 0 || g.batch <= 0 || g.split_k <= 0) return false;
  const bool act = g.mode == EPI_ACT_GELU || g.mode == EPI_ACT_TANH;
  const bool plain = g.mode == EPI_STORE && !g.addf;
  if (a_kc && b_rc && !act) {            // VJP contractions
    if (plain && !g.c_is_f32 && g.split_k == 1) *err = launch_variant<true, false, false, FAST_STORE>(g, s);
    else if (g.mode == EPI_MUL_AUX && !g.addf && !g.c_is_f32) *err = launch_variant<true, false, false, FAST_MUL_AUX>(g, s);
    else if (g.mode == EPI_MUL_1MZ2 && !g.addf && !g.c_is_f32) *err = launch_variant<true, false, false, FAST_MUL_1MZ2>(g, s);
    else if (g.mode == EPI_ADD_AUX && !g.addf && !g.c_is_f32) *err = launch_variant<true, false, false, FAST_ADD_AUX>(g, s);
    else *err = launch_variant<true, false, false, FAST_NONE>(g, s);
  } else if (a_rc && b_rc && !act) {     // parameter gradients
    if (plain && (g.c_is_f32 || g.split_k > 1)) *err = launch_variant<false, false, false, FAST_STORE_F32>(g, s);
    else *err = launch_variant<false, false, false, FAST_NONE>(g, s);
  } else if (a_kc && b_kc) {             // forward
    *err = act ? launch_variant<true, true, true, FAST_NONE>(g, s) : launch_variant<true, true, false, FAST_NONE>(g, s);
  } else {
    return false;
  }
  return true;
}

}  // namespace hbp
