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

constexpr int BM = 256, BK = 32;
constexpr int A_BYTES = BM * BK * 2;            // 16 KB
// WN = wave columns of the workgroup: 2 -> tile 256 x 128, 4 waves, 3 stages, two
// workgroups per CU; 4 -> tile 256 x 256, 8 waves, 4 stages, one workgroup per CU.
template <int WN> struct Cfg {
  static constexpr int BN = 64 * WN;
  static constexpr int NW = 2 * WN;                 // waves
  static constexpr int NTHR = 64 * NW;
  static constexpr int NST = WN == 2 ? 3 : 4;
  static constexpr int B_BYTES = BN * BK * 2;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int MIN_WG = WN == 2 ? 2 : 1;    // workgroups per CU
};
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
template <bool KC, int ROWS, int NW>
struct TileSrc {
  static constexpr int NI = ROWS / 16 / NW;     // copies per wave per slice
  static constexpr int CH = ROWS / 8;           // RC: 16-byte chunks per k row
  const bf16_t* p[NI];                          // pointer at slice 0 (may be out of range: guarded by ok/klim)
  bool ok[NI];                                  // the fixed coordinate is inside the matrix
  int kofs[NI];                                 // k offset of this lane's chunk within a slice
  long step;                                    // elements per slice

  __device__ __forceinline__ void init(const bf16_t* base, long ld, long row0, long rows_lim, long k_begin,
                                       int wave, int lane) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int j = wave + NW * i;              // copy index within the tile: 1 KB each
      if (KC) {
        const int r = 16 * j + (lane >> 2);
        const int c = (lane & 3) ^ ((r >> 2) & 3);
        ok[i] = row0 + r < rows_lim;
        kofs[i] = 8 * c;
        p[i] = base + (row0 + r) * ld + k_begin + 8 * c;
      } else {
        constexpr int KPI = 64 / CH;            // k rows per copy
        const int k = j * KPI + lane / CH;
        const int c = (lane % CH) ^ (4 * (k & 3));
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
      dma16(src, lds_tile + (unsigned)(wave + NW * i) * 1024u);
    }
  }
};

// 32 rows x 16 k fragment: lane l holds row (l % 32), k = kk + 8*(l/32) .. +7
template <bool KC, int ROWS>
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

template <bool A_KC, bool B_KC, int WN>
__global__ __launch_bounds__(Cfg<WN>::NTHR, Cfg<WN>::MIN_WG) void gemm_mfma_kernel(GemmArgs g, int tiles_m,
                                                                                   int tiles_n, long total,
                                                                                   long per_xcd) {
  typedef Cfg<WN> C;
  constexpr int BN = C::BN, NST = C::NST, STAGE_BYTES = C::STAGE_BYTES;
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
  const int wm0 = (wave / WN) * 128, wn0 = (wave % WN) * 64;
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

  TileSrc<A_KC, BM, C::NW> sa;
  TileSrc<B_KC, BN, C::NW> sb;
  sa.init(A, lda, m0, g.M, k_begin, wave, lane);
  sb.init(B, ldb, n0, g.N, k_begin, wave, lane);

  float16v acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // prologue: NST-1 slices in flight
#pragma unroll
  for (int s = 0; s < NST - 1; ++s)
    if (s < KT) {
      sa.issue(s, k_begin, k_end, lds0 + s * STAGE_BYTES, wave, lane);
      sb.issue(s, k_begin, k_end, lds0 + s * STAGE_BYTES + A_BYTES, wave, lane);
    }

  constexpr int PER_SLICE = TileSrc<A_KC, BM, C::NW>::NI + TileSrc<B_KC, BN, C::NW>::NI;  // copies per wave per slice

  // A slice is consumed in four groups of 2 x 2 MFMA blocks (k half, row half).
  // The A fragments of group g+1 are read from LDS while the MFMAs of group g
  // run, and the first fragments of slice kt+1 while the last group of slice kt
  // runs, so the matrix cores do not wait for LDS.
  auto load_b = [&](const unsigned char* bt, bf16x8 (&b)[2][2]) {
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int j = 0; j < 2; ++j) b[h][j] = frag<B_KC, BN>(bt, wn0 + 32 * j, 16 * h, lane);
  };
  auto load_a = [&](const unsigned char* at, int grp, bf16x8 (&a)[2]) {
#pragma unroll
    for (int ii = 0; ii < 2; ++ii) a[ii] = frag<A_KC, BM>(at, wm0 + 32 * ((grp & 1) * 2 + ii), 16 * (grp >> 1), lane);
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
  // waits until at most n slices' worth of this wave's copies are outstanding
  auto wait_slices = [&](int n) {
    if (n >= 2) wait_vm<2 * PER_SLICE>();
    else if (n == 1) wait_vm<PER_SLICE>();
    else wait_vm<0>();
  };

  bf16x8 bcur[2][2], bnxt[2][2], a0[2], a1[2];
  if (KT > 0) {
    wait_slices((KT - 1 < NST - 2 ? KT - 1 : NST - 2));   // slice 0 has landed (this wave's part)
    __syncthreads();                                      // ... and every other wave's
    load_b(smem + A_BYTES, bcur);
    load_a(smem, 0, a0);
  }
  int st = 0;                                  // stage of slice kt
  for (int kt = 0; kt < KT; ++kt) {
    const unsigned char* at = smem + st * STAGE_BYTES;
    load_a(at, 1, a1);
    mma(0, a0, bcur);
    __builtin_amdgcn_sched_barrier(0);
    load_a(at, 2, a0);
    mma(1, a1, bcur);
    __builtin_amdgcn_sched_barrier(0);
    load_a(at, 3, a1);
    mma(2, a0, bcur);
    __builtin_amdgcn_sched_barrier(0);
    int sn = st + 1; if (sn == NST) sn = 0;    // stage of slice kt+1
    if (kt + 1 < KT) {
      // slice kt+1 has landed once only the slices issued after it are outstanding
      const int last = kt + NST - 2 < KT - 1 ? kt + NST - 2 : KT - 1;
      wait_slices(last - (kt + 1));
      __syncthreads();   // every wave's part of slice kt+1 is in LDS; everyone is done reading slice kt-1
      if (kt + NST - 1 < KT) {
        int sf = st + NST - 1; if (sf >= NST) sf -= NST;   // stage of slice kt-1: free now
        sa.issue(kt + NST - 1, k_begin, k_end, lds0 + sf * STAGE_BYTES, wave, lane);
        sb.issue(kt + NST - 1, k_begin, k_end, lds0 + sf * STAGE_BYTES + A_BYTES, wave, lane);
      }
      const unsigned char* an = smem + sn * STAGE_BYTES;
      load_b(an + A_BYTES, bnxt);
      load_a(an, 0, a0);
    }
    mma(3, a1, bcur);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int j = 0; j < 2; ++j) bcur[h][j] = bnxt[h][j];
    st = sn;
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

template <bool A_KC, bool B_KC, int WN>
hipError_t launch_variant(const GemmArgs& g, hipStream_t s) {
  typedef Cfg<WN> C;
  constexpr int BN = C::BN, NTHR = C::NTHR;
  constexpr size_t lds_main = (size_t)C::NST * C::STAGE_BYTES;
  constexpr size_t lds_epi = (size_t)C::NW * EPI_WAVE * sizeof(float);
  constexpr size_t lds_bytes = lds_main > lds_epi ? lds_main : lds_epi;
  static bool attr_set = false;
  auto kern = gemm_mfma_kernel<A_KC, B_KC, WN>;
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
  // Long contractions take the 256 x 256 tile (fewest bytes through L2 per
  // flop); short ones, where the epilogue weighs as much as the main loop, the
  // 256 x 128 tile with two workgroups per CU overlapping each other.
  const bool wide = g.tile_hint ? g.tile_hint == 4 : (g.K / g.split_k >= 1024 && g.N > 128);
  if (a_kc && b_rc) *err = wide ? launch_variant<true, false, 4>(g, s) : launch_variant<true, false, 2>(g, s);
  else if (a_rc && b_rc) *err = wide ? launch_variant<false, false, 4>(g, s) : launch_variant<false, false, 2>(g, s);
  else if (a_kc && b_kc) *err = wide ? launch_variant<true, true, 4>(g, s) : launch_variant<true, true, 2>(g, s);
  else return false;
  return true;
}

}  // namespace hbp
