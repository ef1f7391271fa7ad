// Shared device helpers and the internal launcher interface of libhbp.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hbp {

typedef unsigned short bf16_t;  // raw bf16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t h) {
  return __uint_as_float(((unsigned int)h) << 16);
}
// round to nearest, ties to even (inputs here are finite)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  unsigned int u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// two floats -> two bf16 in one word, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ unsigned int pack_bf16x2(float a, float b) {
  typedef float f2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 b2_t __attribute__((ext_vector_type(2)));
  const f2_t v = {a, b};
  return __builtin_bit_cast(unsigned int, __builtin_convertvector(v, b2_t));
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// 8 consecutive elements <-> 8 floats (16-byte accesses for bf16, 2 x 16 for fp32)
__device__ __forceinline__ void load8(const bf16_t* p, float (&o)[8]) {
  uint4 r = *reinterpret_cast<const uint4*>(p);
  unsigned int w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    o[2 * i] = __uint_as_float(w[i] << 16);
    o[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
  }
}
__device__ __forceinline__ void load8(const float* p, float (&o)[8]) {
  float4 a = *reinterpret_cast<const float4*>(p);
  float4 b = *reinterpret_cast<const float4*>(p + 4);
  o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
  o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}
__device__ __forceinline__ void store8(bf16_t* p, const float (&v)[8]) {
  unsigned int w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) w[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
  *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
}
__device__ __forceinline__ void store8(float* p, const float (&v)[8]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}

// store8 with a non-temporal hint
__device__ __forceinline__ void store8_nt(bf16_t* p, const float (&v)[8]) {
  typedef unsigned u4 __attribute__((ext_vector_type(4)));
  u4 w;
#pragma unroll
  for (int i = 0; i < 4; ++i) w[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
  __builtin_nontemporal_store(w, reinterpret_cast<u4*>(p));
}
__device__ __forceinline__ void store8_nt(float* p, const float (&v)[8]) {
  typedef float f4 __attribute__((ext_vector_type(4)));
  const f4 a = {v[0], v[1], v[2], v[3]}, b = {v[4], v[5], v[6], v[7]};
  __builtin_nontemporal_store(a, reinterpret_cast<f4*>(p));
  __builtin_nontemporal_store(b, reinterpret_cast<f4*>(p + 4));
}

// 8 consecutive elements as loaded, unpacked later: lets a kernel issue a batch
// of loads before it touches any of the values.
template <typename T> struct Raw8;
template <> struct Raw8<bf16_t> {
  uint4 v;
  __device__ __forceinline__ void load(const bf16_t* p) { v = *reinterpret_cast<const uint4*>(p); }
  // streamed once: non-temporal (does not displace what other kernels keep in the caches)
  __device__ __forceinline__ void load_nt(const bf16_t* p) {
    typedef unsigned u4 __attribute__((ext_vector_type(4)));
    const u4 t = __builtin_nontemporal_load(reinterpret_cast<const u4*>(p));
    v = make_uint4(t.x, t.y, t.z, t.w);
  }
  __device__ __forceinline__ void unpack(float (&o)[8]) const {
    const unsigned int w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      o[2 * i] = __uint_as_float(w[i] << 16);
      o[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
  }
};
template <> struct Raw8<float> {
  float4 a, b;
  __device__ __forceinline__ void load(const float* p) {
    a = *reinterpret_cast<const float4*>(p);
    b = *reinterpret_cast<const float4*>(p + 4);
  }
  __device__ __forceinline__ void load_nt(const float* p) {
    typedef float f4 __attribute__((ext_vector_type(4)));
    const f4 t = __builtin_nontemporal_load(reinterpret_cast<const f4*>(p));
    const f4 u = __builtin_nontemporal_load(reinterpret_cast<const f4*>(p + 4));
    a = make_float4(t.x, t.y, t.z, t.w);
    b = make_float4(u.x, u.y, u.z, u.w);
  }
  __device__ __forceinline__ void unpack(float (&o)[8]) const {
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
    o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
  }
};

// ---------------------------------------------------------------------------
// GEMM:  C[b][m,n] = epilogue( sum_k A[b](m,k) * B[b](k,n) )
// ---------------------------------------------------------------------------
enum EpiMode {
  EPI_STORE = 0,       // C = acc
  EPI_MUL_AUX = 1,     // C = acc * aux[m,n]                    (da = dz * act'(a))
  EPI_MUL_1MZ2 = 2,    // C = acc * (1 - aux[m,n]^2)            (tanh: aux = z)
  EPI_ACT_GELU = 3,    // C = gelu(acc); out2 = gelu'(acc)
  EPI_ACT_TANH = 4,    // C = tanh(acc)
  EPI_RESID = 5,       // C = lambda[n] * aux[m,n] + acc        (x_{l+1})
  EPI_ADD_AUX = 6      // C = acc + aux[m,n]
};

struct GemmArgs {
  const void* A; const void* B; void* C;
  long M, N, K;
  long a_sm, a_sk;      // element strides of A(m,k)
  long b_sk, b_sn;      // element strides of B(k,n)
  long ldc;             // row stride of C, aux, out2, addf
  long batch;           // grid.z
  long a_sb, b_sb, c_sb;  // batch strides (elements)
  int split_k;          // >1: C is fp32 partials [split][batch][M,N] (EPI_STORE only)
  int mode;
  const void* aux; long aux_sb;       // storage type
  void* out2; long out2_sb;           // storage type
  const float* addf; long addf_sb;    // fp32 [M,N], added to acc before the epilogue
  const float* lambda; long lambda_sb;  // fp32 [N]
  const void* lambda_mn;              // storage type [M,N] (row stride ldc, batch stride aux_sb): EPI_RESID per element
  int c_is_f32;         // C stored as fp32 regardless of the storage type
};

// storage type: 0 = fp32, 1 = bf16
hipError_t launch_gemm_generic(int dtype, const GemmArgs& g, hipStream_t s);
// fast bf16 MFMA path; returns false when the shape/layout is not covered
bool launch_gemm_mfma(const GemmArgs& g, hipStream_t s, hipError_t* err);

// Multi-head self-attention on rows [q | k | v] (3 d wide, head h in columns h dh .. of each third), `seqs` sequences of
// T consecutive rows each; o and dout are d wide.  lse and dsum hold one float per (sequence, head, position).
struct AttnArgs {
  const void* qkv;      // storage type [seqs * T, 3 d]
  void* o;              // forward: out; backward: in   [seqs * T, d]
  float* lse;           // forward: out; backward: in   log2 of each row's sum of exp2(s log2 e)
  const void* dout;     // backward: gradient of o      [seqs * T, d]
  void* dqkv;           // backward: out                [seqs * T, 3 d]
  float* dsum;          // backward: scratch            sum_c dout (.) o per row and head
  long seqs, T;
  int heads, dh, causal;
  float scale;          // 1 / sqrt(dh)
  int by_problem;       // set by the launchers: how workgroup ids map to (problem, block of tiles)
};
bool attn_supported(int dtype, long T, int dh);
hipError_t launch_attn_fwd(int dtype, const AttnArgs& a, hipStream_t s);
hipError_t launch_attn_bwd(int dtype, const AttnArgs& a, hipStream_t s);

// Few-row bf16 product with both operands K-contiguous: C[M,N] = epilogue(A[M,K] . Bt[N,K]^T).
// Modes EPI_STORE, EPI_ACT_TANH, EPI_MUL_AUX, EPI_MUL_1MZ2, EPI_ADD_AUX; aux is bf16 [M,N] with row stride ldaux.
// EPI_RESID here is the residual path's backward step, C = acc (+ aux) + lambda (.) next: next and
// lambda_mn are bf16 [M,N] with C's row stride, lambda is fp32 [N]; neither lambda given means 1.
struct SkinnyArgs {
  const void* A; long lda;
  const void* Bt; long ldbt;
  void* C; long ldc;
  long M, N, K;
  int mode;
  const void* aux; long ldaux;
  const void* next;
  const float* lambda;
  const void* lambda_mn;
  const float* addf;   // fp32 [M,N] with C's row stride, added to the product before the epilogue; or NULL
  int c_is_f32;        // C stored as fp32 (EPI_STORE only)
};
bool skinny_ok(long M, long N, long K);   // M <= 128, N % 32 == 0, K % 64 == 0
hipError_t launch_gemm_skinny(const SkinnyArgs& a, hipStream_t s);
// dst[cols,rows] = src[rows,cols]^T, 2-byte elements
hipError_t launch_transpose_bf16(const void* src, void* dst, int rows, int cols, hipStream_t s);

// out[i] = sum_s part[s][i], i < n
hipError_t launch_splitk_reduce(const float* part, float* out, long n, int split, hipStream_t s);

// ---------------------------------------------------------------------------
// residual-path scan:  for l = l_hi-1 .. l_lo:
//   v_l = has_v ? (norm ? rmsnorm_bwd(dn_l; y_l, rinv_l) : dn_l) : 0
//   g_l = (e_l) + v_l + res_gamma lambda_l (.) g_{l+1}^{old} + (1 - res_gamma') lambda_l (.) g_{l+1}
// (written below as blk_gamma and res_scale).  g[l_hi] must already hold the
// incoming state gradient; g^{old} is what g held before this scan.
// ---------------------------------------------------------------------------
struct ScanArgs {
  void* g;              // [L+1,N,d] storage
  const void* dn;       // [L,N,d] storage (block input gradient before the norm's backward), or NULL
  const void* y;        // [L,N,d] storage (RMS only)
  const float* rinv;    // [L,N]   (RMS only)
  const void* e;        // [L+1,N,d] storage or NULL
  const float* lambda;  // [L,d] or NULL
  const void* lambda_tok;  // [L,N,d] storage, or NULL: coefficients per token (then lambda is NULL)
  long N, d;
  long l_lo, l_hi;
  int norm_rms;
  float* chunk_ws;      // scratch of scan_chunk_ws_bytes() for the chunked form (long chains), or NULL
  int force;            // 0: the launcher picks the form; 1: the sequential form; 2: the chunked three-pass form;
                        // 3: the single-pass form (2 and 3 need chunk_ws; 3: bf16, one value stream, no old-estimate term)
  float res_scale;      // factor on lambda along the residual path (1 - gamma; 1 for the plain method)
  float blk_gamma;      // gamma: adds gamma lambda_l (.) g_{l+1}^{old} to v_l (0: nothing read)
  const uint8_t* mask;  // [L,N,d/8] bits or NULL: g_l (l >= 1) is multiplied by the bits of row block l-1 (the ReLU
                        // that made x_l) before it is stored and carried on; direct forms only, gamma = 0
};
hipError_t launch_scan(int dtype, const ScanArgs& a, hipStream_t s);
// Long chains with few of them (the time axis of an RNN) are cut into chunks of
// SCAN_CHUNK states scanned in parallel; bytes of fp32 scratch that form needs
// (0 when the direct form is used).
constexpr long SCAN_CHUNK = 64;
size_t scan_chunk_ws_bytes(long L, long N, long d, int norm_rms);
size_t scan_chunk_ws_bytes_forced(long L, long N, long d);   // the same when the chunked form is asked for by name
size_t scan_sp_ws_bytes(long L, long N, long d, int lambda_tok);   // scratch of the single-pass form (force = 3)

// The scan in the form of the paper's Algorithm 1 (Hillis-Steele): ceil(log2(L+1)) sweeps over all
// positions, each adding the partner 2^s positions up, in fp32 scratch.  Kept for comparison: it
// moves O(L log L) elements where the forms above move O(L).  u_i = a_i + lambda_i (.) u_{i+1}.
struct HsArgs {
  void* g;              // out [L+1,N,d] storage
  const void* e;        // a: [L+1,N,d] storage (every_state) or [N,d] (a_L only, the rest 0)
  int every_state;
  const float* lambda;  // [L,d] or NULL
  const void* lambda_tok;  // [L,N,d] storage or NULL
  float res_scale;
  long L, N, d;
  float* ws;            // hs_ws_bytes()
};
size_t hs_ws_bytes(long L, long N, long d, int lambda_kind);   // 0 one, 1 channel, 2 token
hipError_t launch_scan_hillis_steele(int dtype, const HsArgs& a, hipStream_t s);

// The residual-path scan of a post-norm stack (x_{l+1} = RMSnorm(lambda_l (.) x_l + block_l(x_l))); g holds the
// state gradients taken through the norm that made each state.  See scan_post_kernel.
struct PostScanArgs {
  void* g;              // [L+1,N,d] storage
  const void* dn;       // [L,N,d] storage: block input gradients (with e_l already added when e is NULL), or NULL
  const void* e;        // [L+1,N,d] storage or NULL: added per state
  const void* e_top;    // [N,d] storage: e_L (modes 0 and 2)
  const void* x;        // [L+1,N,d] storage: the (normalised) states
  const float* lambda;  // [L,d] or NULL
  const float* rho;     // [L,N]: 1/rms of the sums
  const float* m_old;   // [L,N]: mean(G_{l+1} (.) x_{l+1}) of the previous estimate (mode 0 with dn)
  float* m_new;         // [L,N]: the same of this one
  long N, d;
  long l_lo, l_hi;      // mode 0: layers l_hi-1 .. l_lo with l_hi = L; mode 1: the one layer l_lo (l_hi = l_lo + 1);
  int mode;             // mode 2: l_hi = L, no layer
  float gamma;          // mode 0: the residual path is scaled by 1 - gamma
  float blk_gamma;      // mode 0: gamma lambda_l (.) g[l+1]^{old} is added to the block term (0: the old g is not read)
};
hipError_t launch_scan_post(int dtype, const PostScanArgs& a, hipStream_t s);
hipError_t launch_rmsnorm_inplace(int dtype, void* x, float* rinv, long rows, long d, float eps, hipStream_t s);

// x := max(x, 0) over n elements (n % 8 == 0), mask bit = 1 where x was positive; g := g (.) mask bits
hipError_t launch_relu_mask(int dtype, void* x, uint8_t* mask, long n, hipStream_t s);
hipError_t launch_mask_apply(int dtype, void* g, const uint8_t* mask, long n, hipStream_t s);

// The gated recurrent cell's elementwise parts (H % 8 == 0): one step forward from pre [N,2H] fp32, and step (i)
// up to its contraction for `rows` token rows of consecutive blocks (g points at the gradient of block 0's NEXT state).
hipError_t launch_gated_fwd(int dtype, const float* pre, const void* x, void* uc, void* a, void* xn, long N, long H,
                            hipStream_t s);
hipError_t launch_gated_vjp(int dtype, const void* g, const void* x, const void* uc, void* da, long rows, long H,
                            hipStream_t s);

// The standard GRU's elementwise parts (gates kept as zrn = [z | r | n] [.,3H]; H % 8 == 0): the two halves of a step
// forward (pre [N,3H] fp32), and of step (i) for `rows` token rows (see gated_cell.hip).
hipError_t launch_gru_fwd1(int dtype, const float* pre, const void* x, void* zrn, void* rx, long N, long H, hipStream_t s);
hipError_t launch_gru_fwd2(int dtype, const float* pre, const void* x, void* zrn, void* a, void* xn, long N, long H,
                           hipStream_t s);
hipError_t launch_gru_vjp1(int dtype, const void* g, const void* x, const void* zrn, void* da, long rows, long H,
                           hipStream_t s);
hipError_t launch_gru_vjp2(int dtype, void* drx, const void* x, const void* zrn, const void* e, void* da, void* rx,
                           long rows, long H, hipStream_t s);

// The LSTM cell's elementwise parts (state [c | h] of width 2H, gates [i | f | o | gg] of width 4H, H % 8 == 0):
// one step forward from pre [N,4H] fp32; step (i) up to its contraction for `rows` token rows (g: gradient of the
// rows' next states, x / xn: current / next states, e: per-state loss gradients whose cell half is added to v, or NULL).
hipError_t launch_lstm_fwd(int dtype, const float* pre, const void* x, void* gates, void* a, void* xn, long N, long H,
                           hipStream_t s);
hipError_t launch_lstm_vjp(int dtype, const void* g, const void* x, const void* xn, const void* gates, const void* e,
                           void* da, void* v, long rows, long H, hipStream_t s);

// ---------------------------------------------------------------------------
// the training step around the backward pass (train.hip)
// ---------------------------------------------------------------------------
struct OptimArgs {
  float lr, beta1 /* SGD: momentum */, beta2, eps, weight_decay;
  float inv_bias1, inv_bias2;     // AdamW: 1 / (1 - beta^step)
};
size_t train_scratch_floats();    // floats of scratch the reductions below need
// e = (x - target) * inv_n over n elements (n % 8 == 0), loss[0] = 0.5 * inv_n * sum (x - target)^2
hipError_t launch_mse_loss_grad(int dtype, const void* x, const void* target, void* e, long n, float inv_n,
                                float* scratch, float* loss, hipStream_t s);
hipError_t launch_zero(int dtype, void* p, long n, hipStream_t s);   // n % 8 == 0
hipError_t launch_clip_factor(const float* const* grads, const long* sizes, int count, float max_norm, float* scratch,
                              float* factor, hipStream_t s);
hipError_t launch_optim(int dtype, int adamw, void* w, float* master, const float* g, float* m, float* v, long n,
                        const float* clip, const OptimArgs& o, hipStream_t s);

// y = x * rinv, rinv = 1/sqrt(mean(x^2)+eps) for `rows` rows of width d
hipError_t launch_rmsnorm_fwd(int dtype, const void* x, void* y, float* rinv, long rows, long d, float eps,
                              hipStream_t s);

}  // namespace hbp
