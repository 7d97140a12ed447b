// GEMM family: C[M,N] = op(A) op(B) (+bias) (+res), optional gelu second output,
// fp32 accumulate-into-C for weight gradients.
//
//  * k_gemm_mfma: bf16 operands on the gfx950 matrix cores
//    (v_mfma_f32_32x32x16_bf16), 128x128 block tile, four wavefronts each owning
//    a 64x64 sub-tile (2x2 MFMA tiles, 64 fp32 accumulators per lane), K tiles of
//    64 staged through double-buffered, XOR-swizzled LDS with the next tile's
//    global loads in flight during the current tile's MFMAs.  Operands whose
//    contraction index is NOT the contiguous one (dgrad's W, wgrad's dY and X) are
//    transposed on their way into LDS (4x8 register patches, 8-byte stores), so
//    the inner loop is the same for every layout.  Accumulating GEMMs with few
//    output tiles split the contraction over workgroups (fp32 atomics).
//  * k_gemm_ref: plain 64x64 tiled fp32-FMA kernel for any layout and element
//    type; the fp32 precision path and the A/B reference for the MFMA kernel.
#include <algorithm>

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
  int c_fp32, accumulate, res_fp32;
};

// ---- shared epilogue ---------------------------------------------------------
template <typename E>
__device__ __forceinline__ void epilogue_store(const GemmP &p, int m, int n, float v) {
  if (p.bias) v += to_f32(static_cast<const E *>(p.bias)[n]);
  if (p.res)
    v += p.res_fp32 ? static_cast<const float *>(p.res)[int64_t(m) * p.ldr + n]
                    : to_f32(static_cast<const E *>(p.res)[int64_t(m) * p.ldr + n]);
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
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int TILE_ELEMS = BM * BK;   // 16 KiB per operand per stage; 2 operands x 2 stages = 64 KiB

// LDS holds every operand tile as [row][k] with 128-byte rows whose eight 16-byte
// chunks are XOR-swizzled by the row, so that both the 16-byte MFMA fragment reads
// (16 consecutive rows, one chunk) and the 8-byte transposing stores spread over
// all banks.
__device__ __forceinline__ int lds_swz(int row) { return ((row >> 1) ^ (row >> 4)) & 7; }
__device__ __forceinline__ int lds_addr(int row, int k) {   // in elements
  return row * BK + ((((k >> 3) ^ lds_swz(row)) & 7) << 3) + (k & 7);
}

// Global -> registers for one 128(row) x 64(k) operand tile; 4 x 16 bytes per thread.
// TR = false: memory is [row][k]: chunk q = tid + 256 i covers row q/8, k (q%8)*8..+7.
// TR = true : memory is [k][row]: thread owns rows (tid%16)*8..+7 at k (tid/16)*4 + i.
// Branch-free: addresses are clamped into the operand (the leading dimension covers
// the contiguous extent rounded up to 8, checked by the launcher).  Rows beyond the
// operand are NOT zeroed: they only feed output rows/columns that are never stored.
// Only the K tail (last tile, uniform branch) is zeroed, on packed 32-bit words.
template <bool TR>
struct TileLoader {
  const bf16_t *base;
  uint32_t ld;
  int K, kpart;
  uint32_t off[TR ? 1 : 4];     // element offsets that do not depend on k
  __device__ __forceinline__ void init(const bf16_t *b, int64_t ld_, int row0, int nrows, int K_, int tid) {
    base = b; ld = uint32_t(ld_); K = K_;
    if (!TR) {
      kpart = (tid % 8) * 8;
#pragma unroll
      for (int i = 0; i < 4; ++i) off[i] = uint32_t(min(row0 + (tid + 256 * i) / 8, nrows - 1)) * ld;
    } else {
      kpart = (tid / 16) * 4;
      off[0] = uint32_t(min(row0 + (tid % 16) * 8, ((nrows + 7) & ~7) - 8));
    }
  }
  __device__ __forceinline__ void load(int kt, Vec16<bf16_t> (&r)[4]) const {
    const int k0 = kt * BK;
    const bool tail = k0 + BK > K;
    if (!TR) {
      const int gk = k0 + kpart;
      const uint32_t gkc = uint32_t(min(gk, ((K + 7) & ~7) - 8));
#pragma unroll
      for (int i = 0; i < 4; ++i) r[i] = load16(base + (off[i] + gkc));
      if (tail) {
        const int nv = K - gk;    // valid elements of this thread's chunks (same k range for all four)
        uint32_t mask[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) mask[w] = nv >= 2 * w + 2 ? 0xffffffffu : (nv == 2 * w + 1 ? 0x0000ffffu : 0u);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          uint32_t *u = reinterpret_cast<uint32_t *>(&r[i]);
#pragma unroll
          for (int w = 0; w < 4; ++w) u[w] &= mask[w];
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t gkc = uint32_t(min(k0 + kpart + i, K - 1));
        r[i] = load16(base + (gkc * ld + off[0]));
      }
      if (tail) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const uint32_t keep = (k0 + kpart + i < K) ? 0xffffffffu : 0u;
          uint32_t *u = reinterpret_cast<uint32_t *>(&r[i]);
#pragma unroll
          for (int w = 0; w < 4; ++w) u[w] &= keep;
        }
      }
    }
  }
};
template <bool TR>
__device__ __forceinline__ void store_tile_lds(bf16_t *s, int tid, const Vec16<bf16_t> (&r)[4]) {
  if (!TR) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int q = tid + 256 * i;
      store16(s + lds_addr(q / 8, (q % 8) * 8), r[i]);
    }
  } else {
    // registers hold a 4(k) x 8(row) patch; write it transposed, 4 k-values (8 bytes) per row
    const int row_base = (tid % 16) * 8, k = (tid / 16) * 4;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      bf16x4 t;
      t[0] = r[0].v[j]; t[1] = r[1].v[j]; t[2] = r[2].v[j]; t[3] = r[3].v[j];
      *reinterpret_cast<bf16x4 *>(s + lds_addr(row_base + j, k)) = t;
    }
  }
}
// MFMA operand fragment: 8 consecutive k of one row, 16 bytes
__device__ __forceinline__ bf16x8 load_frag(const bf16_t *s, int row, int k) {
  return *reinterpret_cast<const bf16x8 *>(s + lds_addr(row, k));
}

// One K tile from LDS in two halves: eight 16-byte fragments (one exposed LDS
// latency), then their eight MFMAs back to back.
__device__ __forceinline__ void mma_tile(const bf16_t *a_s, const bf16_t *b_s, int arow, int brow, int kg,
                                         f32x16 (&acc)[2][2]) {
#pragma unroll
  for (int half = 0; half < BK / 32; ++half) {
    bf16x8 fa[2][2], fb[2][2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        fa[ks][i] = load_frag(a_s, arow + i * 32, (half * 2 + ks) * 16 + kg);
        fb[ks][i] = load_frag(b_s, brow + i * 32, (half * 2 + ks) * 16 + kg);
      }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks][i], fb[ks][j], acc[i][j], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
}

template <bool TA, bool TB>
__global__ __launch_bounds__(256, 2) void k_gemm_mfma(GemmP p, int tiles_per_split, int grid_n) {
  __shared__ __attribute__((aligned(16))) bf16_t sA[2][TILE_ELEMS];
  __shared__ __attribute__((aligned(16))) bf16_t sB[2][TILE_ELEMS];
  const bf16_t *A = static_cast<const bf16_t *>(p.A), *B = static_cast<const bf16_t *>(p.B);
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  const int wm = wave / 2, wn = wave % 2;
  // Tile order.  Consecutive workgroup ids go round-robin over the 8 XCDs (each with its
  // own L2), so first give each XCD a contiguous range of tile ids; then walk the tile
  // grid in bands of 8 tile rows, column by column, so that the ~64 workgroups resident
  // on an XCD form an 8x8 patch that shares 8 row panels of A and 8 column panels of B
  // in L2 instead of streaming one whole operand per tile row.
  int bid = blockIdx.x;
  const int nb = gridDim.x, grid_m = nb / grid_n;
  if (nb % 8 == 0) bid = (bid % 8) * (nb / 8) + bid / 8;
  constexpr int kBand = 8;
  const int band = bid / (kBand * grid_n), first_m = band * kBand;
  const int band_rows = min(grid_m - first_m, kBand);
  const int in_band = bid - band * kBand * grid_n;
  const int m0 = (first_m + in_band % band_rows) * BM, n0 = (in_band / band_rows) * BN;
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk_all = (p.K + BK - 1) / BK;
  const int kt0 = blockIdx.y * tiles_per_split;
  const int kt1 = min(nk_all, kt0 + tiles_per_split);
  const int arow = wm * 64 + lane % 32, brow = wn * 64 + lane % 32, kg = (lane / 32) * 8;
  // Software pipeline: while tile kt is multiplied out of LDS stage kt&1, tile kt+1 is
  // in flight from HBM into registers; it is stored to the other stage after the MFMAs.
  Vec16<bf16_t> ra[4], rb[4];
  TileLoader<TA> la;
  TileLoader<TB> lb;
  la.init(A, p.lda, m0, p.M, p.K, tid);
  lb.init(B, p.ldb, n0, p.N, p.K, tid);
  if (kt0 < kt1) {
    la.load(kt0, ra);
    lb.load(kt0, rb);
    store_tile_lds<TA>(sA[0], tid, ra);
    store_tile_lds<TB>(sB[0], tid, rb);
  }
  __syncthreads();
  for (int kt = kt0; kt < kt1; ++kt) {
    const int cur = (kt - kt0) & 1;
    if (kt + 1 < kt1) {
      la.load(kt + 1, ra);
      lb.load(kt + 1, rb);
    }
    mma_tile(sA[cur], sB[cur], arow, brow, kg, acc);
    if (kt + 1 < kt1) {
      store_tile_lds<TA>(sA[cur ^ 1], tid, ra);
      store_tile_lds<TB>(sB[cur ^ 1], tid, rb);
    }
    __syncthreads();
  }
  // accumulator layout of the 32x32 MFMA: register r of lane l holds
  // row 8*(r/4) + 4*(l/32) + r%4, column l%32
  const bool split = gridDim.y > 1;
  int m_base = m0 + wm * 64 + 4 * (lane / 32), n_base = n0 + wn * 64 + lane % 32;
  // keep the 64 output addresses from being computed (and kept live) before the main loop
  asm volatile("" : "+v"(m_base), "+v"(n_base));
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int n = n_base + j * 32;
    if (n >= p.N) continue;
    const float bias_v = p.bias ? to_f32(static_cast<const bf16_t *>(p.bias)[n]) : 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m_base + i * 32 + 8 * (r / 4) + r % 4;
        if (m >= p.M) continue;
        const int64_t ci = int64_t(m) * p.ldc + n;
        float v = acc[i][j][r] + bias_v;
        if (p.res)
          v += p.res_fp32 ? static_cast<const float *>(p.res)[int64_t(m) * p.ldr + n]
                          : to_f32(static_cast<const bf16_t *>(p.res)[int64_t(m) * p.ldr + n]);
        if (split) {
          atomicAdd(static_cast<float *>(p.C) + ci, v);   // C += partial
        } else if (p.c_fp32) {
          float *c = static_cast<float *>(p.C);
          c[ci] = p.accumulate ? c[ci] + v : v;
        } else {
          const bf16_t o = from_f32<bf16_t>(v);
          static_cast<bf16_t *>(p.C)[ci] = o;
          if (p.gelu_out) static_cast<bf16_t *>(p.gelu_out)[ci] = from_f32<bf16_t>(gelu_f(to_f32(o)));
        }
      }
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
  if (g.res_fp32 && g.res && !g.c_fp32) return fail(HMY_E_INVALID, "gemm: an fp32 residual needs an fp32 C");
  const int64_t min_lda = g.ta ? g.M : g.K, min_ldb = g.tb ? g.N : g.K;
  if (g.lda < min_lda || g.ldb < min_ldb || g.ldc < g.N || (g.res && g.ldr < g.N))
    return fail(HMY_E_INVALID, "gemm: leading dimension too small");
  GemmP p;
  p.A = g.A; p.B = g.B; p.C = g.C; p.bias = g.bias; p.res = g.res; p.gelu_out = g.gelu_out;
  p.M = g.M; p.N = g.N; p.K = g.K;
  p.lda = g.lda; p.ldb = g.ldb; p.ldc = g.ldc; p.ldr = g.ldr;
  p.c_fp32 = g.c_fp32; p.accumulate = g.accumulate;
  p.res_fp32 = g.res_fp32 || g.prec == HMY_PREC_FP32;
  hipStream_t s = (hipStream_t)st;
  // 32-bit element offsets inside the kernel: every operand must span fewer than 2^31 elements
  const int64_t a_span = int64_t(g.ta ? g.K : g.M) * g.lda, b_span = int64_t(g.tb ? g.K : g.N) * g.ldb;
  const bool mfma_ok = g.prec == HMY_PREC_BF16 && g_use_mfma && aligned16(g.A) && aligned16(g.B) && g.lda % 8 == 0 &&
                       g.ldb % 8 == 0 && a_span < (int64_t(1) << 31) && b_span < (int64_t(1) << 31);
  if (mfma_ok && g_use_mfma == 1 && gemm_dma_eligible(g)) return launch_gemm_dma(g, st);
  if (mfma_ok && g_use_mfma == 1 && g.K % 32 != 0 && g.K > 256 && g.accumulate && g.c_fp32 && !g.bias && !g.res) {
    // accumulating GEMM with a ragged contraction: the multiple-of-32 part goes to the
    // load-to-LDS kernel, the tail is added by the register-staged one (which masks)
    hmy_gemm_desc body = g, tail = g;
    body.K = g.K / 32 * 32;
    tail.K = g.K - body.K;
    tail.A = static_cast<const bf16_t *>(g.A) + (g.ta ? int64_t(body.K) * g.lda : int64_t(body.K));
    tail.B = static_cast<const bf16_t *>(g.B) + (g.tb ? int64_t(body.K) * g.ldb : int64_t(body.K));
    if (gemm_dma_eligible(body) && aligned16(tail.A) && aligned16(tail.B)) {
      const int rc = launch_gemm_dma(body, st);
      return rc ? rc : launch_gemm_mfma32(tail, st);
    }
  }
  if (mfma_ok && g_use_mfma != 2) return launch_gemm_mfma32(g, st);
  if (mfma_ok) {
    const int gm = (g.M + BM - 1) / BM, gn = (g.N + BN - 1) / BN, nk = (g.K + BK - 1) / BK;
    // split the contraction over workgroups (fp32 atomics into C) when an accumulating
    // GEMM has too few output tiles to fill 256 compute units
    int splits = 1;
    if (g.accumulate && g.c_fp32 && !g.bias && !g.res && gm * gn < 512)
      splits = std::max(1, std::min((768 + gm * gn - 1) / (gm * gn), nk / 4));
    const int tiles_per_split = (nk + splits - 1) / splits;
    splits = (nk + tiles_per_split - 1) / tiles_per_split;
    dim3 grid(gm * gn, splits), block(256);
    if (!g.ta && !g.tb) hipLaunchKernelGGL((k_gemm_mfma<false, false>), grid, block, 0, s, p, tiles_per_split, gn);
    else if (!g.ta && g.tb) hipLaunchKernelGGL((k_gemm_mfma<false, true>), grid, block, 0, s, p, tiles_per_split, gn);
    else if (g.ta && !g.tb) hipLaunchKernelGGL((k_gemm_mfma<true, false>), grid, block, 0, s, p, tiles_per_split, gn);
    else hipLaunchKernelGGL((k_gemm_mfma<true, true>), grid, block, 0, s, p, tiles_per_split, gn);
    return check_launch("gemm_mfma");
  }
  // bf16 operands that the matrix-core kernels cannot take (not 16-byte aligned, or a leading dimension that is
  // not a multiple of 8 elements) are an error while those kernels are selected: the plain kernel below would be
  // tens of times slower, and nobody would be told
  if (g.prec == HMY_PREC_BF16 && g_use_mfma)
    return fail(HMY_E_INVALID, "gemm: bf16 operands must be 16-byte aligned with leading dimensions that are multiples "
                               "of 8 elements (lda %lld, ldb %lld) and span less than 2^31 elements",
                (long long)g.lda, (long long)g.ldb);
  const int64_t a_sm = g.ta ? 1 : g.lda, a_sk = g.ta ? g.lda : 1;
  const int64_t b_sn = g.tb ? 1 : g.ldb, b_sk = g.tb ? g.ldb : 1;
  dim3 grid((g.N + 63) / 64, (g.M + 63) / 64), block(256);
  if (g.prec == HMY_PREC_FP32) hipLaunchKernelGGL(k_gemm_ref<float>, grid, block, 0, s, p, a_sm, a_sk, b_sn, b_sk);
  else hipLaunchKernelGGL(k_gemm_ref<bf16_t>, grid, block, 0, s, p, a_sm, a_sk, b_sn, b_sk);
  return check_launch("gemm_ref");
}

}  // namespace hmy
