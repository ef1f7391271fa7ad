// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32
// accumulate) for the VJP and parameter-gradient contractions.
//
// One workgroup of 8 wavefronts (2 x 4) owns a 256 x 256 output tile; each
// wavefront a 128 x 64 sub-tile = 4 x 2 MFMA blocks of 32 x 32 (128 accumulator
// registers per lane).  The contraction runs in slices of 64, double-buffered
// in LDS: while the MFMAs consume slice t, the global loads of slice t+1 are
// in flight in registers.
//
// An operand tile sits in LDS in the orientation it has in memory:
//   KC  contraction index contiguous  [256 rows][64 k]  -> a lane's 8 k-values
//       are one 16-byte ds_read;
//   RC  row index contiguous          [64 k][256 rows]  -> the lane's 8 k-values
//       are strided, fetched with the LDS transpose read ds_read_b64_tr_b16
//       (two per fragment).  Within a group of 16 lanes that instruction gives
//       lane j element r = element (j % 4) of the 8 bytes addressed by lane
//       4*r + j/4, i.e. a 4 x 16 transpose.
// The three pairings cover every contraction of the path:
//   NN (A KC, B RC)  da = g W2,  dn = da W1           (weights read as stored)
//   TN (A RC, B RC)  dW2 = g^T z, dW1 = da^T y, dU    (contraction over tokens)
//   NT (A KC, B KC)  forward  a = y W1^T, out = z W2^T
// Rows/columns beyond the matrix are loaded as zeros and not stored, so any
// size with the contiguous dimensions a multiple of 8 is covered.
//
// Epilogue: the accumulators go through a wave-private LDS buffer so that every
// global access of the epilogue (output, and the element-wise operand it is
// fused with) is a 16-byte row-contiguous access.
//
// Workgroup -> tile mapping: consecutive workgroup ids are dealt round-robin to
// the 8 XCDs, each with its own L2, so id % 8 selects a contiguous eighth of
// the tile list and the tiles one XCD works on at a time share operand panels.
#include "hbp_common.h"

namespace hbp {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int BM = 256, BN = 256, BK = 64, NTHR = 512;
constexpr int KC_LD = BK + 8;          // 72 elements = 144 B: 8 consecutive rows hit 32 distinct banks
constexpr int RC_LD = 256 + 16;        // 272 elements = 544 B: 4 consecutive k rows hit disjoint bank octets
constexpr int KC_TILE = 256 * KC_LD;   // elements
constexpr int RC_TILE = BK * RC_LD;
constexpr int EPI_LD = 64 + 4;         // floats per staged row
constexpr int EPI_WAVE = 32 * EPI_LD;  // floats per wave

template <bool KC>
__device__ __forceinline__ void gload(const bf16_t* __restrict__ base, long ld, long row0, long rows_lim, long k0,
                                      long k_lim, int tid, uint4 (&r)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = tid + NTHR * i;
    long row, k;
    const bf16_t* p;
    if (KC) {
      row = row0 + (c >> 3);
      k = k0 + 8 * (c & 7);
      p = base + row * ld + k;
    } else {
      k = k0 + (c >> 5);
      row = row0 + 8 * (c & 31);
      p = base + k * ld + row;
    }
    if (row < rows_lim && k < k_lim)
      r[i] = *reinterpret_cast<const uint4*>(p);
    else
      r[i] = make_uint4(0u, 0u, 0u, 0u);
  }
}

template <bool KC>
__device__ __forceinline__ void sstore(bf16_t* tile, int tid, const uint4 (&r)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = tid + NTHR * i;
    bf16_t* p = KC ? tile + (c >> 3) * KC_LD + 8 * (c & 7) : tile + (c >> 5) * RC_LD + 8 * (c & 31);
    *reinterpret_cast<uint4*>(p) = r[i];
  }
}

// 32 rows x 16 k fragment: lane l holds row (l % 32), k = 8*(l/32) .. +7
template <bool KC>
__device__ __forceinline__ bf16x8 frag(const bf16_t* tile, int row0, int k0, int lane) {
  if (KC) {
    const bf16_t* p = tile + (row0 + (lane & 31)) * KC_LD + k0 + 8 * (lane >> 5);
    uint4 v = *reinterpret_cast<const uint4*>(p);
    return __builtin_bit_cast(bf16x8, v);
  } else {
    const int s = lane & 15;
    const bf16_t* p = tile + (k0 + 8 * (lane >> 5) + (s >> 2)) * RC_LD + row0 + 16 * ((lane >> 4) & 1) + 4 * (s & 3);
    typedef __attribute__((address_space(3))) short4v* lds_p;
    short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p));
    short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p + 4 * RC_LD));
    short8v v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
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
__global__ __launch_bounds__(NTHR) void gemm_mfma_kernel(GemmArgs g, int tiles_m, int tiles_n, long total, long per_xcd) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int A_TILE = A_KC ? KC_TILE : RC_TILE;
  constexpr int B_TILE = B_KC ? KC_TILE : RC_TILE;
  bf16_t* lds = reinterpret_cast<bf16_t*>(smem);
  bf16_t* As[2] = {lds, lds + A_TILE + B_TILE};
  bf16_t* Bs[2] = {lds + A_TILE, lds + 2 * A_TILE + B_TILE};

  // XCD-aware tile id
  const long bid = blockIdx.x;
  const long t = (bid & 7) * per_xcd + (bid >> 3);
  if (t >= total) return;
  const long tiles_mn = (long)tiles_m * tiles_n;
  const long zb = t / tiles_mn;            // batch * split_k + split
  const long rem = t - zb * tiles_mn;
  const int tm = (int)(rem / tiles_n), tn = (int)(rem % tiles_n);
  const long batch = zb / g.split_k;
  const int split = (int)(zb % g.split_k);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave >> 2) * 128, wn0 = (wave & 3) * 64;
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

  float16v acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  uint4 ra[4], rb[4];
  if (KT > 0) {
    gload<A_KC>(A, lda, m0, g.M, k_begin, k_end, tid, ra);
    gload<B_KC>(B, ldb, n0, g.N, k_begin, k_end, tid, rb);
    sstore<A_KC>(As[0], tid, ra);
    sstore<B_KC>(Bs[0], tid, rb);
  }
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < KT) {
      const long k0 = k_begin + (long)(kt + 1) * BK;
      gload<A_KC>(A, lda, m0, g.M, k0, k_end, tid, ra);
      gload<B_KC>(B, ldb, n0, g.N, k0, k_end, tid, rb);
    }
    const bf16_t* at = As[cur];
    const bf16_t* bt = Bs[cur];
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
      bf16x8 af[4], bfr[2];
#pragma unroll
      for (int i = 0; i < 4; ++i) af[i] = frag<A_KC>(at, wm0 + 32 * i, kk, lane);
#pragma unroll
      for (int j = 0; j < 2; ++j) bfr[j] = frag<B_KC>(bt, wn0 + 32 * j, kk, lane);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) {
      sstore<A_KC>(As[cur ^ 1], tid, ra);
      sstore<B_KC>(Bs[cur ^ 1], tid, rb);
    }
    __syncthreads();
  }

  // ---- epilogue: stage 32 rows at a time through wave-private LDS ----
  float* stage = reinterpret_cast<float*>(smem) + wave * EPI_WAVE;
  const int er = lane >> 3;         // row within a group of 8
  const int ec = (lane & 7) * 8;    // first of 8 columns
  const long col = n0 + wn0 + ec;
  const bool col_ok = col < g.N;
  const float* lam = g.lambda ? g.lambda + batch * g.lambda_sb : nullptr;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
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
      const bf16_t* aux = reinterpret_cast<const bf16_t*>(g.aux) + batch * g.aux_sb + off;
      switch (g.mode) {
        case EPI_MUL_AUX: {
          float t8[8];
          load8(aux, t8);
#pragma unroll
          for (int x = 0; x < 8; ++x) v[x] *= t8[x];
          break;
        }
        case EPI_MUL_1MZ2: {
          float t8[8];
          load8(aux, t8);
#pragma unroll
          for (int x = 0; x < 8; ++x) v[x] *= (1.f - t8[x] * t8[x]);
          break;
        }
        case EPI_ACT_GELU: {
          float d8[8];
#pragma unroll
          for (int x = 0; x < 8; ++x) { d8[x] = gelu_grad_f(v[x]); v[x] = gelu_f(v[x]); }
          store8(reinterpret_cast<bf16_t*>(g.out2) + batch * g.out2_sb + off, d8);
          break;
        }
        case EPI_ACT_TANH: {
#pragma unroll
          for (int x = 0; x < 8; ++x) v[x] = tanhf(v[x]);
          break;
        }
        case EPI_RESID: {
          float t8[8];
          load8(aux, t8);
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
        }
        case EPI_ADD_AUX: {
          float t8[8];
          load8(aux, t8);
#pragma unroll
          for (int x = 0; x < 8; ++x) v[x] += t8[x];
          break;
        }
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
  constexpr int A_TILE = A_KC ? KC_TILE : RC_TILE;
  constexpr int B_TILE = B_KC ? KC_TILE : RC_TILE;
  constexpr size_t lds_main = (size_t)2 * (A_TILE + B_TILE) * sizeof(bf16_t);
  constexpr size_t lds_epi = (size_t)8 * EPI_WAVE * sizeof(float);
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
