// GEMM family: C[M,N] = op(A) op(B) (+bias) (+res), optional gelu second output,
// fp32 accumulate-into-C for weight gradients.
//
//  * k_gemm_mfma: bf16 operands on the gfx950 matrix cores
//    (v_mfma_f32_32x32x16_bf16), 128x128 block tile, four wavefronts each owning
//    a 64x64 sub-tile (2x2 MFMA tiles, 64 fp32 accumulators per lane), K tiles of
//    32 staged through double-buffered LDS with the next tile's global loads in
//    flight during the current tile's MFMAs.  Operands whose contraction index
//    is NOT the contiguous one (dgrad's W, wgrad's dY and X) are stored in LDS
//    as loaded and gathered per lane.
//  * k_gemm_ref: plain 64x64 tiled fp32-FMA kernel for any layout and element
//    type; the fp32 precision path and the A/B reference for the MFMA kernel.
#include "dev_common.h"
#include "hmy_internal.h"

namespace hmy {

int g_use_mfma = 1;

namespace {

struct GemmP {
  const void *A, *B;
  void *C;
  const void *bias, *res;
  void *gelu_out;
  int M, N, K;
  int64_t lda, ldb, ldc, ldr;
  int c_fp32, accumulate;
};

// ---- shared epilogue ---------------------------------------------------------
template <typename E>
__device__ __forceinline__ void epilogue_store(const GemmP &p, int m, int n, float v) {
  if (p.bias) v += to_f32(static_cast<const E *>(p.bias)[n]);
  if (p.res) v += to_f32(static_cast<const E *>(p.res)[int64_t(m) * p.ldr + n]);
  const int64_t ci = int64_t(m) * p.ldc + n;
  if (p.c_fp32) {
    float *c = static_cast<float *>(p.C);
    c[ci] = p.accumulate ? c[ci] + v : v;
  } else {
    const E r = from_f32<E>(v);
    static_cast<E *>(p.C)[ci] = r;
    if (p.gelu_out) static_cast<E *>(p.gelu_out)[ci] = from_f32<E>(gelu_f(to_f32(r)));
  }
}

// ---- reference kernel ------------------------------------------------------------
template <typename E>
__global__ __launch_bounds__(256) void k_gemm_ref(GemmP p, int64_t a_sm, int64_t a_sk, int64_t b_sn, int64_t b_sk) {
  constexpr int BT = 64, BK = 16, PAD = 4;
  __shared__ __attribute__((aligned(16))) float sA[BK][BT + PAD];
  __shared__ __attribute__((aligned(16))) float sB[BK][BT + PAD];
  const E *A = static_cast<const E *>(p.A), *B = static_cast<const E *>(p.B);
  const int m0 = blockIdx.y * BT, n0 = blockIdx.x * BT;
  const int tid = threadIdx.x, ty = tid / 16, tx = tid % 16;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < p.K; k0 += BK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = tid + i * 256;
      int m, k;
      if (a_sk == 1) { k = idx % BK; m = idx / BK; } else { m = idx % BT; k = idx / BT; }
      const int gm = m0 + m, gk = k0 + k;
      sA[k][m] = (gm < p.M && gk < p.K) ? to_f32(A[gm * a_sm + gk * a_sk]) : 0.f;
      int n, kb;
      if (b_sk == 1) { kb = idx % BK; n = idx / BK; } else { n = idx % BT; kb = idx / BT; }
      const int gn = n0 + n, gkb = k0 + kb;
      sB[kb][n] = (gn < p.N && gkb < p.K) ? to_f32(B[gn * b_sn + gkb * b_sk]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      const float4 a = *reinterpret_cast<const float4 *>(&sA[kk][ty * 4]);
      const float4 b = *reinterpret_cast<const float4 *>(&sB[kk][tx * 4]);
      const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < p.M && n < p.N) epilogue_store<E>(p, m, n, acc[i][j]);
    }
}

// ---- MFMA kernel -----------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 32;
constexpr int PITCH_K = BK + 8;    // [row][k] layout: 80-byte rows, conflict-free 16-byte reads
constexpr int PITCH_T = BM + 8;    // [k][row] layout for operands stored contraction-major
constexpr int TILE_ELEMS = (BM * PITCH_K > BK * PITCH_T) ? BM * PITCH_K : BK * PITCH_T;

// Load this thread's two 16-byte chunks of a 128(row) x 32(k) operand tile.
// TR = false: memory is [row][k] (k contiguous).  TR = true: memory is [k][row].
// Out-of-range elements are zero.
template <bool TR>
__device__ __forceinline__ void load_tile_regs(const bf16_t *base, int64_t ld, int row0, int k0, int nrows, int K, int tid,
                                               Vec16<bf16_t> (&r)[2]) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    int row, k, n_valid;
    if (!TR) {
      row = tid / 4 + 64 * i;
      k = (tid % 4) * 8;
      const int gr = row0 + row, gk = k0 + k;
      n_valid = (gr < nrows) ? min(8, K - gk) : 0;
      const bf16_t *src = base + int64_t(gr) * ld + gk;
      if (n_valid >= 8) {
        r[i] = load16(src);
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) r[i].v[j] = (j < n_valid) ? src[j] : bf16_t(0.f);
      }
    } else {
      k = tid / 16 + 16 * i;
      row = (tid % 16) * 8;
      const int gr = row0 + row, gk = k0 + k;
      n_valid = (gk < K) ? min(8, nrows - gr) : 0;
      const bf16_t *src = base + int64_t(gk) * ld + gr;
      if (n_valid >= 8) {
        r[i] = load16(src);
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) r[i].v[j] = (j < n_valid) ? src[j] : bf16_t(0.f);
      }
    }
  }
}
template <bool TR>
__device__ __forceinline__ void store_tile_lds(bf16_t *s, int tid, const Vec16<bf16_t> (&r)[2]) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    if (!TR) {
      const int row = tid / 4 + 64 * i, k = (tid % 4) * 8;
      store16(s + row * PITCH_K + k, r[i]);
    } else {
      const int k = tid / 16 + 16 * i, row = (tid % 16) * 8;
      store16(s + k * PITCH_T + row, r[i]);
    }
  }
}
// MFMA operand fragment: lane holds 8 consecutive k of row (row0 + lane%32), k group lane/32.
template <bool TR>
__device__ __forceinline__ bf16x8 load_frag(const bf16_t *s, int row, int k) {
  if (!TR) {
    return *reinterpret_cast<const bf16x8 *>(s + row * PITCH_K + k);
  } else {
    bf16x8 f;
#pragma unroll
    for (int j = 0; j < 8; ++j) f[j] = s[(k + j) * PITCH_T + row];
    return f;
  }
}

template <bool TA, bool TB>
__global__ __launch_bounds__(256) void k_gemm_mfma(GemmP p) {
  __shared__ __attribute__((aligned(16))) bf16_t sA[2][TILE_ELEMS];
  __shared__ __attribute__((aligned(16))) bf16_t sB[2][TILE_ELEMS];
  const bf16_t *A = static_cast<const bf16_t *>(p.A), *B = static_cast<const bf16_t *>(p.B);
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  const int wm = wave / 2, wn = wave % 2;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  Vec16<bf16_t> ra[2], rb[2];
  const int nk = (p.K + BK - 1) / BK;
  load_tile_regs<TA>(A, p.lda, m0, 0, p.M, p.K, tid, ra);
  load_tile_regs<TB>(B, p.ldb, n0, 0, p.N, p.K, tid, rb);   // tb=1: B is stored [K][N]
  store_tile_lds<TA>(sA[0], tid, ra);
  store_tile_lds<TB>(sB[0], tid, rb);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) {
      load_tile_regs<TA>(A, p.lda, m0, (kt + 1) * BK, p.M, p.K, tid, ra);
      load_tile_regs<TB>(B, p.ldb, n0, (kt + 1) * BK, p.N, p.K, tid, rb);
    }
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const int k = ks * 16 + (lane / 32) * 8;
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) fa[i] = load_frag<TA>(sA[cur], wm * 64 + i * 32 + lane % 32, k);
#pragma unroll
      for (int j = 0; j < 2; ++j) fb[j] = load_frag<TB>(sB[cur], wn * 64 + j * 32 + lane % 32, k);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) {
      store_tile_lds<TA>(sA[cur ^ 1], tid, ra);
      store_tile_lds<TB>(sB[cur ^ 1], tid, rb);
    }
    __syncthreads();
  }
  // accumulator layout of the 32x32 MFMA: register r of lane l holds
  // row 8*(r/4) + 4*(l/32) + r%4, column l%32
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * 64 + i * 32 + 8 * (r / 4) + 4 * (lane / 32) + r % 4;
        const int n = n0 + wn * 64 + j * 32 + lane % 32;
        if (m < p.M && n < p.N) epilogue_store<bf16_t>(p, m, n, acc[i][j][r]);
      }
}

inline int check_launch(const char *what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(HMY_E_HIP, "launch of %s failed: %s", what, hipGetErrorString(e));
  return HMY_OK;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

int launch_gemm(const hmy_gemm_desc &g, stream_t st) {
  if (g.M < 1 || g.N < 1 || g.K < 1) return fail(HMY_E_INVALID, "gemm: empty shape %dx%dx%d", g.M, g.N, g.K);
  if (!g.A || !g.B || !g.C) return fail(HMY_E_INVALID, "gemm: null operand");
  if (g.accumulate && !g.c_fp32) return fail(HMY_E_INVALID, "gemm: accumulate needs an fp32 C");
  if (g.gelu_out && g.c_fp32) return fail(HMY_E_INVALID, "gemm: gelu output needs an element-typed C");
  if (g.prec != HMY_PREC_FP32 && g.prec != HMY_PREC_BF16) return fail(HMY_E_INVALID, "gemm: unknown precision");
  const int64_t min_lda = g.ta ? g.M : g.K, min_ldb = g.tb ? g.N : g.K;
  if (g.lda < min_lda || g.ldb < min_ldb || g.ldc < g.N || (g.res && g.ldr < g.N))
    return fail(HMY_E_INVALID, "gemm: leading dimension too small");
  GemmP p;
  p.A = g.A; p.B = g.B; p.C = g.C; p.bias = g.bias; p.res = g.res; p.gelu_out = g.gelu_out;
  p.M = g.M; p.N = g.N; p.K = g.K;
  p.lda = g.lda; p.ldb = g.ldb; p.ldc = g.ldc; p.ldr = g.ldr;
  p.c_fp32 = g.c_fp32; p.accumulate = g.accumulate;
  hipStream_t s = (hipStream_t)st;
  const bool mfma_ok = g.prec == HMY_PREC_BF16 && g_use_mfma && aligned16(g.A) && aligned16(g.B) && g.lda % 8 == 0 &&
                       g.ldb % 8 == 0;
  if (mfma_ok) {
    dim3 grid((g.N + BN - 1) / BN, (g.M + BM - 1) / BM), block(256);
    if (!g.ta && !g.tb) hipLaunchKernelGGL((k_gemm_mfma<false, false>), grid, block, 0, s, p);
    else if (!g.ta && g.tb) hipLaunchKernelGGL((k_gemm_mfma<false, true>), grid, block, 0, s, p);
    else if (g.ta && !g.tb) hipLaunchKernelGGL((k_gemm_mfma<true, false>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((k_gemm_mfma<true, true>), grid, block, 0, s, p);
    return check_launch("gemm_mfma");
  }
  const int64_t a_sm = g.ta ? 1 : g.lda, a_sk = g.ta ? g.lda : 1;
  const int64_t b_sn = g.tb ? 1 : g.ldb, b_sk = g.tb ? g.ldb : 1;
  dim3 grid((g.N + 63) / 64, (g.M + 63) / 64), block(256);
  if (g.prec == HMY_PREC_FP32) hipLaunchKernelGGL(k_gemm_ref<float>, grid, block, 0, s, p, a_sm, a_sk, b_sn, b_sk);
  else hipLaunchKernelGGL(k_gemm_ref<bf16_t>, grid, block, 0, s, p, a_sm, a_sk, b_sn, b_sk);
  return check_launch("gemm_ref");
}

}  // namespace hmy
