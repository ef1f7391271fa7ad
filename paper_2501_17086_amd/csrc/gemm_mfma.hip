// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32
// accumulate) for the VJP and parameter-gradient contractions.
//
// Shape of the kernel
//   workgroup   4 wavefronts (2 x 2), output tile 256 x 128; a wavefront owns
//               128 x 64 = 4 x 2 MFMA blocks of 32 x 32 (128 accumulator
//               registers per lane).  Two workgroups are resident per CU, each
//               with its own barriers, so one's epilogue and barrier stalls
//               overlap the other's MFMA work.
//   K pipeline  slices of 32, three LDS stages per workgroup (72 KB); slices
//               are copied global -> LDS directly (global_load_lds_dwordx4, no
//               staging registers), two slices ahead of the one being
//               multiplied, one barrier per slice.
//   LDS layout  an operand tile sits in LDS in the orientation it has in memory:
//                 KC  contraction index contiguous, [rows][32 k]: a lane's 8
//                     k-values are one 16-byte ds_read;
//                 RC  row index contiguous, [32 k][rows]: the lane's 8 k-values
//                     are strided and fetched with the LDS transpose read
//                     ds_read_b64_tr_b16 (two per fragment; within 16 lanes it
//                     returns to lane j, element r, element j%4 of the 8 bytes
//                     addressed by lane 4r + j/4).
//               A direct-to-LDS copy writes 1 KB per wavefront contiguously, so
//               rows cannot be padded; bank conflicts are avoided by an XOR
//               swizzle of the 16-byte chunk index instead, applied on the
//               global-address side of the copy and again by the readers.
//   pairings    NN (A KC, B RC)  da = g W2, dn = da W1   (weights as stored)
//               TN (A RC, B RC)  dW2 = g^T z, dW1 = da^T y, dU
//               NT (A KC, B KC)  forward  a = y W1^T, out = z W2^T
//   edges       chunks outside the matrix are copied from a zero-filled device
//               array, rows/columns outside are not stored: any size whose
//               contiguous dimensions are multiples of 8 is covered.
//   epilogue    accumulators pass through wave-private LDS so that every global
//               access (output and the fused element-wise operand) is a
//               16-byte row-contiguous access; the fused operand of the next 32
//               rows is fetched while the current 32 are processed.
//   tile order  workgroup ids are dealt round-robin to the 8 XCDs (one L2
//               each): id % 8 selects a contiguous eighth of the tile list, and
//               the list walks 8 x 8 blocks of tiles so that the tiles an XCD
//               works on at one time share operand panels.
#include "hbp_common.h"

namespace hbp {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int BM = 256, BN = 128, BK = 32, NST = 3, NTHR = 256;
constexpr int A_BYTES = BM * BK * 2;            // 16 KB
constexpr int B_BYTES = BN * BK * 2;            //  8 KB
constexpr int STAGE_BYTES = A_BYTES + B_BYTES;  // 24 KB
constexpr int EPI_LD = 64 + 4;                  // floats per staged row
constexpr int EPI_WAVE = 32 * EPI_LD;           // floats per wave
constexpr int GROUP_M = 8;                      // tile rows per block of the tile walk

__device__ uint4 g_zero_chunks[64];  // source of out-of-range chunks (zero-initialised)

// 16 bytes per lane, global -> LDS at lds_base + lane * 16.  lds_base is
// wave-uniform.  The compiler does not see this write to LDS: callers order it
// against LDS reads with wait_vm() + __syncthreads().
__device__ __forceinline__ void dma16(const void* gptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off\n"
               :: "v"(gptr), "s"(lds_base) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vm() {   // at most N vector-memory loads outstanding
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// Per-lane source description of one operand tile's copies (ROWS/64 per wave).
template <bool KC, int ROWS>
struct TileSrc {
  static constexpr int NI = ROWS / 64;          // copies per wave per slice
  static constexpr int CH = ROWS / 8;           // RC: 16-byte chunks per k row
  const bf16_t* p[NI];                          // pointer at slice 0 (may be out of range: guarded by ok/klim)
  bool ok[NI];                                  // the fixed coordinate is inside the matrix
  int kofs[NI];                                 // k offset of this lane's chunk within a slice
  long step;                                    // elements per slice

  __device__ __forceinline__ void init(const bf16_t* base, long ld, long row0, long rows_lim, long k_begin,
                                       int wave, int lane) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int j = wave + 4 * i;               // copy index within the tile: 1 KB each
      if (KC) {
        const int r = 16 * j + (lane >> 2);
        const int c = (lane & 3) ^ ((r >> 1) & 3);
        ok[i] = row0 + r < rows_lim;
        kofs[i] = 8 * c;
        p[i] = base + (row0 + r) * ld + k_begin + 8 * c;
      } else {
        constexpr int KPI = 64 / CH;            // k rows per copy
        const int k = j * KPI + lane / CH;
        const int c = (lane % CH) ^ (2 * (k & 3));
        ok[i] = row0 + 8 * c < rows_lim;
        kofs[i] = k;
        p[i] = base + (k_begin + k) * ld + row0 + 8 * c;
      }
    }
    step = KC ? BK : BK * ld;
  }
  // copies slice t (k range starts at k_begin + t*BK) into the tile at LDS byte address lds_tile
  __device__ __forceinline__ void issue(int t, long k_begin, long k_end, unsigned lds_tile, int wave, int lane) const {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const bool v = ok[i] && (k_begin + (long)t * BK + kofs[i] < k_end);
      const void* src = v ? (const void*)(p[i] + (long)t * step) : (const void*)(g_zero_chunks + lane);
      dma16(src, lds_tile + (unsigned)(wave + 4 * i) * 1024u);
    }
  }
};

// 32 rows x 16 k fragment: lane l holds row (l % 32), k = kk + 8*(l/32) .. +7
template <bool KC, int ROWS>
__device__ __forceinline__ bf16x8 frag(const unsigned char* tile, int row0, int kk, int lane) {
  if (KC) {
    const int r = row0 + (lane & 31);
    const int c = (kk >> 3) + (lane >> 5);
    const uint4 v = *reinterpret_cast<const uint4*>(tile + r * 64 + ((c ^ ((r >> 1) & 3)) << 4));
    return __builtin_bit_cast(bf16x8, v);
  } else {
    typedef __attribute__((address_space(3))) short4v* lds_p;
    const int s = lane & 15;
    const int e = row0 + 16 * ((lane >> 4) & 1) + 4 * (s & 3);
    const int k = kk + 8 * (lane >> 5) + (s >> 2);          // k & 3 == s >> 2 for both halves
    const int sw = 2 * (s >> 2);
    const unsigned char* p = tile + k * (ROWS * 2) + (((e >> 3) ^ sw) << 4) + (e & 7) * 2;
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p + 4 * (ROWS * 2)));
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

template <bool A_KC, bool B_KC>
__global__ __launch_bounds__(NTHR, 2) void gemm_mfma_kernel(GemmArgs g, int tiles_m, int tiles_n, long total,
                                                            long per_xcd) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

  // ---- XCD-aware tile id, walking 8 x 8 blocks of tiles ----
  const long bid = blockIdx.x;
  const long t = (bid & 7) * per_xcd + (bid >> 3);
  if (t >= total) return;
  const long tiles_mn = (long)tiles_m * tiles_n;
  const long zb = t / tiles_mn;            // batch * split_k + split
  const long rem = t - zb * tiles_mn;
  const long grp = rem / ((long)GROUP_M * tiles_n);
  const long in_grp = rem - grp * GROUP_M * tiles_n;
  const int gm = (int)((tiles_m - grp * GROUP_M) < GROUP_M ? (tiles_m - grp * GROUP_M) : GROUP_M);
  const int tm = (int)(grp * GROUP_M + in_grp % gm), tn = (int)(in_grp / gm);
  const long batch = zb / g.split_k;
  const int split = (int)(zb % g.split_k);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave >> 1) * 128, wn0 = (wave & 1) * 64;
  const long m0 = (long)tm * BM, n0 = (long)tn * BN;

  const bf16_t* A = reinterpret_cast<const bf16_t*>(g.A) + batch * g.a_sb;
  const bf16_t* B = reinterpret_cast<const bf16_t*>(g.B) + batch * g.b_sb;
  const long lda = A_KC ? g.a_sm : g.a_sk;
  const long ldb = B_KC ? g.b_sn : g.b_sk;

  long kchunk = (g.K + g.split_k - 1) / g.split_k;
  kchunk = (kchunk + BK - 1) / BK * BK;
  const long k_begin = (long)split * kchunk;
  long k_end = k_begin + kchunk;
  if (k_end > g.K) k_end = g.K;
  const int KT = k_end > k_begin ? (int)((k_end - k_begin + BK - 1) / BK) : 0;

  const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;

  TileSrc<A_KC, BM> sa;
  TileSrc<B_KC, BN> sb;
  sa.init(A, lda, m0, g.M, k_begin, wave, lane);
  sb.init(B, ldb, n0, g.N, k_begin, wave, lane);

  float16v acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // prologue: two slices in flight
#pragma unroll
  for (int s = 0; s < NST - 1; ++s)
    if (s < KT) {
      sa.issue(s, k_begin, k_end, lds0 + s * STAGE_BYTES, wave, lane);
      sb.issue(s, k_begin, k_end, lds0 + s * STAGE_BYTES + A_BYTES, wave, lane);
    }

  constexpr int PER_SLICE = TileSrc<A_KC, BM>::NI + TileSrc<B_KC, BN>::NI;  // copies per wave per slice
  int st = 0;                                  // stage of slice kt
  for (int kt = 0; kt < KT; ++kt) {
    // slice kt has landed once at most the copies of slice kt+1 are still outstanding
    if (kt + 1 < KT) wait_vm<PER_SLICE>(); else wait_vm<0>();
    __syncthreads();                           // ... for every wave; and everyone is done reading slice kt-1
    if (kt + NST - 1 < KT) {
      int sn = st + NST - 1; if (sn >= NST) sn -= NST;   // stage of slice kt-1: free now
      sa.issue(kt + NST - 1, k_begin, k_end, lds0 + sn * STAGE_BYTES, wave, lane);
      sb.issue(kt + NST - 1, k_begin, k_end, lds0 + sn * STAGE_BYTES + A_BYTES, wave, lane);
    }
    const unsigned char* at = smem + st * STAGE_BYTES;
    const unsigned char* bt = at + A_BYTES;
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
      bf16x8 af[4], bfr[2];
#pragma unroll
      for (int i = 0; i < 4; ++i) af[i] = frag<A_KC, BM>(at, wm0 + 32 * i, kk, lane);
#pragma unroll
      for (int j = 0; j < 2; ++j) bfr[j] = frag<B_KC, BN>(bt, wn0 + 32 * j, kk, lane);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (++st == NST) st = 0;
  }
  __syncthreads();   // all waves are done with the operand stages before they are reused below

  // ---- epilogue: 32 rows at a time through wave-private LDS ----
  float* stage = reinterpret_cast<float*>(smem) + wave * EPI_WAVE;
  const int er = lane >> 3;         // row within a group of 8
  const int ec = (lane & 7) * 8;    // first of 8 columns
  const long col = n0 + wn0 + ec;
  const bool col_ok = col < g.N;
  const float* lam = g.lambda ? g.lambda + batch * g.lambda_sb : nullptr;
  const bool use_aux = g.split_k == 1 && (g.mode == EPI_MUL_AUX || g.mode == EPI_MUL_1MZ2 || g.mode == EPI_RESID ||
                                          g.mode == EPI_ADD_AUX);
  const bf16_t* aux = reinterpret_cast<const bf16_t*>(g.aux) + batch * g.aux_sb;

  uint4 auxv[2][4];
  auto fetch_aux = [&](int i, uint4 (&dst)[4]) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const long row = m0 + wm0 + 32 * i + er + 8 * q;
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
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        stage[row * EPI_LD + j * 32 + (lane & 31)] = acc[i][j][r];
      }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int rr = er + 8 * q;
      const long row = m0 + wm0 + 32 * i + rr;
      float v[8];
      {
        const float4 lo = *reinterpret_cast<const float4*>(stage + rr * EPI_LD + ec);
        const float4 hi = *reinterpret_cast<const float4*>(stage + rr * EPI_LD + ec + 4);
        v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w;
        v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
      }
      if (row >= g.M || !col_ok) continue;
      const long off = row * g.ldc + col;
      if (g.split_k > 1) {
        float* P = reinterpret_cast<float*>(g.C) + ((long)split * g.batch + batch) * g.c_sb + off;
        store8(P, v);
        continue;
      }
      if (g.addf) {
        float t8[8];
        load8(g.addf + batch * g.addf_sb + off, t8);
#pragma unroll
        for (int x = 0; x < 8; ++x) v[x] += t8[x];
      }
      float t8[8];
      {
        const uint4 a4 = auxv[i & 1][q];
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
        case EPI_ACT_GELU: {
          float d8[8];
#pragma unroll
          for (int x = 0; x < 8; ++x) { d8[x] = gelu_grad_f(v[x]); v[x] = gelu_f(v[x]); }
          store8(reinterpret_cast<bf16_t*>(g.out2) + batch * g.out2_sb + off, d8);
          break;
        }
        case EPI_ACT_TANH:
#pragma unroll
          for (int x = 0; x < 8; ++x) v[x] = tanhf(v[x]);
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
        store8(reinterpret_cast<float*>(g.C) + batch * g.c_sb + off, v);
      else
        store8(reinterpret_cast<bf16_t*>(g.C) + batch * g.c_sb + off, v);
    }
    __builtin_amdgcn_wave_barrier();
  }
}

template <bool A_KC, bool B_KC>
hipError_t launch_variant(const GemmArgs& g, hipStream_t s) {
  constexpr size_t lds_main = (size_t)NST * STAGE_BYTES;
  constexpr size_t lds_epi = (size_t)4 * EPI_WAVE * sizeof(float);
  constexpr size_t lds_bytes = lds_main > lds_epi ? lds_main : lds_epi;
  static bool attr_set = false;
  auto kern = gemm_mfma_kernel<A_KC, B_KC>;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int tiles_m = (int)((g.M + BM - 1) / BM), tiles_n = (int)((g.N + BN - 1) / BN);
  const long total = (long)tiles_m * tiles_n * g.batch * g.split_k;
  const long per_xcd = (total + 7) / 8;
  hipLaunchKernelGGL(kern, dim3((unsigned)(per_xcd * 8)), dim3(NTHR), lds_bytes, s, g, tiles_m, tiles_n, total,
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
  if (a_kc && b_rc) *err = launch_variant<true, false>(g, s);
  else if (a_rc && b_rc) *err = launch_variant<false, false>(g, s);
  else if (a_kc && b_kc) *err = launch_variant<true, true>(g, s);
  else return false;
  return true;
}

}  // namespace hbp
