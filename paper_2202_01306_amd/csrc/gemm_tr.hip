// bf16 GEMM on the matrix cores, small-K-tile variant: 128x128 block tile, four
// wavefronts of 64x64 (2x2 v_mfma_f32_32x32x16_bf16), K tiles of 32, two tiles in
// flight in registers while a third is multiplied out of double-buffered LDS; 32 KiB
// of LDS and a small register footprint keep several workgroups resident per CU.
//
// LDS layouts.  An operand whose contraction index is contiguous in memory is kept
// [row][k] with its four 16-byte chunks XOR-swizzled by the row.  An operand stored
// contraction-major is kept as loaded, [k][row], chunks swizzled by k, and read
// through ds_read_b64_tr_b16; that read yields the contraction slots of a 16-group
// in the order 4h+0..3, 8+4h+0..3 (h = lane/32), so whenever one operand is read
// this way the other is stored with its 8-byte halves permuted to the same order.
#include <algorithm>

#include "dev_common.h"
#include "hmy_internal.h"

namespace hmy {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BK = 32, NT = 256;   // square block tile BM x BM, K tile, threads
constexpr int TILE_ELEMS = BM * BK;          // 8 KiB per operand per stage

struct BigP {
  const bf16_t *A, *B;
  void *C;
  const bf16_t *bias, *res;
  bf16_t *gelu_out;
  int M, N, K;
  uint32_t lda, ldb;
  int64_t ldc, ldr;
  int c_fp32, accumulate, res_fp32;
};

// element address inside a [row][k] tile (chunks swizzled by the row)
__device__ __forceinline__ int addr_rk(int row, int chunk) { return row * BK + ((chunk ^ ((row >> 2) & 3)) << 3); }
// element address inside a [k][row] tile (16 chunks per k-row, swizzled by k)
__device__ __forceinline__ int addr_kr(int k, int col) {
  return k * BM + ((((col >> 3) ^ ((k & 3) << 2)) & 15) << 3) + (col & 7);
}

// TR = false: memory [row][k]; thread chunk i (of 2): row tid/4 + 64 i, k chunk tid%4.
// TR = true : memory [k][row]; thread chunk i (of 2): k tid/16 + 16 i, rows (tid%16)*8..+7.
// Loads are clamped into the operand; rows outside it only feed outputs never stored.
template <bool TR>
struct Loader {
  const bf16_t *base;
  uint32_t ld;
  int K;
  uint32_t off[TR ? 1 : 2];
  __device__ __forceinline__ void init(const bf16_t *b, uint32_t ld_, int row0, int nrows, int K_, int tid) {
    base = b; ld = ld_; K = K_;
    if (!TR) {
#pragma unroll
      for (int i = 0; i < 2; ++i) off[i] = uint32_t(min(row0 + tid / 4 + 64 * i, nrows - 1)) * ld;
    } else {
      off[0] = uint32_t(min(row0 + (tid % 16) * 8, ((nrows + 7) & ~7) - 8));
    }
  }
  __device__ __forceinline__ void load(int kt, int tid, Vec16<bf16_t> (&r)[2]) const {
    const int k0 = kt * BK;
    const bool tail = k0 + BK > K;
    if (!TR) {
      const int gk = k0 + (tid % 4) * 8;
      const uint32_t gkc = uint32_t(min(gk, ((K + 7) & ~7) - 8));
#pragma unroll
      for (int i = 0; i < 2; ++i) r[i] = load16(base + (off[i] + gkc));
      if (tail) {
        const int nv = K - gk;
        uint32_t mask[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) mask[w] = nv >= 2 * w + 2 ? 0xffffffffu : (nv == 2 * w + 1 ? 0x0000ffffu : 0u);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          uint32_t *u = reinterpret_cast<uint32_t *>(&r[i]);
#pragma unroll
          for (int w = 0; w < 4; ++w) u[w] &= mask[w];
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const uint32_t gkc = uint32_t(min(k0 + tid / 16 + 16 * i, K - 1));
        r[i] = load16(base + (gkc * ld + off[0]));
      }
      if (tail) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          const uint32_t keep = (k0 + tid / 16 + 16 * i < K) ? 0xffffffffu : 0u;
          uint32_t *u = reinterpret_cast<uint32_t *>(&r[i]);
#pragma unroll
          for (int w = 0; w < 4; ++w) u[w] &= keep;
        }
      }
    }
  }
};

// registers -> LDS.  PERM: store the two 8-byte halves of a [row][k] chunk so that a
// 16-byte read returns contraction slots 4h+0..3, 8+4h+0..3.
template <bool TR, bool PERM>
__device__ __forceinline__ void store_lds(bf16_t *s, int tid, const Vec16<bf16_t> (&r)[2]) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    if (TR) {
      const int k = tid / 16 + 16 * i;
      store16(s + addr_kr(k, (tid % 16) * 8), r[i]);
    } else {
      const int row = tid / 4 + 64 * i, chunk = tid % 4;
      if (!PERM) {
        store16(s + addr_rk(row, chunk), r[i]);
      } else {
        const int g = chunk >> 1, e = chunk & 1;
        const uint2 *h = reinterpret_cast<const uint2 *>(&r[i]);
        *reinterpret_cast<uint2 *>(s + addr_rk(row, 2 * g) + 4 * e) = h[0];
        *reinterpret_cast<uint2 *>(s + addr_rk(row, 2 * g + 1) + 4 * e) = h[1];
      }
    }
  }
}

// operand fragment for the 32 MFMA rows/columns starting at tile row row32, k-step ks (16 deep)
template <bool TR>
__device__ __forceinline__ bf16x8 frag(const bf16_t *s, int row32, int ks, int lane) {
  if (!TR) {
    return *reinterpret_cast<const bf16x8 *>(s + addr_rk(row32 + lane % 32, 2 * ks + lane / 32));
  } else {
    const int q = lane % 16, g16 = (lane / 16) % 2, h = lane / 32;
    const int k = 16 * ks + 4 * h + q / 4, col = row32 + 16 * g16 + 4 * (q % 4);
    typedef __attribute__((address_space(3))) short4v *lds_ptr;
    union { short4v s4[2]; bf16x8 b; } u;
    u.s4[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(s + addr_kr(k, col)));
    u.s4[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(s + addr_kr(k + 8, col)));
    return u.b;
  }
}

template <bool TA, bool TB>
__device__ __forceinline__ void mma_tile(const bf16_t *a_s, const bf16_t *b_s, int arow, int brow, int lane,
                                         f32x16 (&acc)[2][2]) {
  bf16x8 fa[BK / 16][2], fb[BK / 16][2];
#pragma unroll
  for (int ks = 0; ks < BK / 16; ++ks)
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      fa[ks][i] = frag<TA>(a_s, arow + 32 * i, ks, lane);
      fb[ks][i] = frag<TB>(b_s, brow + 32 * i, ks, lane);
    }
#pragma unroll
  for (int ks = 0; ks < BK / 16; ++ks)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks][i], fb[ks][j], acc[i][j], 0, 0, 0);
}

template <bool TA, bool TB>
__global__ __launch_bounds__(NT) void k_gemm_mfma32(BigP p, int tiles_per_split, int grid_n) {
  __shared__ __attribute__((aligned(16))) bf16_t sA[2][TILE_ELEMS];
  __shared__ __attribute__((aligned(16))) bf16_t sB[2][TILE_ELEMS];
  constexpr bool PERM = TA || TB;   // some operand comes through the transposing read
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  const int wm = wave / 2, wn = wave % 2;
  // tile order: contiguous tile-id range per XCD, then bands of 8 tile rows walked column by column
  int bid = blockIdx.x;
  const int nb = gridDim.x, grid_m = nb / grid_n;
  if (nb % 8 == 0) bid = (bid % 8) * (nb / 8) + bid / 8;
  constexpr int kBand = 8;
  const int band = bid / (kBand * grid_n), first_m = band * kBand;
  const int band_rows = min(grid_m - first_m, kBand);
  const int in_band = bid - band * kBand * grid_n;
  const int m0 = (first_m + in_band % band_rows) * BM, n0 = (in_band / band_rows) * BM;

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
  const int arow = wm * 64, brow = wn * 64;
  Loader<TA> la;
  Loader<TB> lb;
  la.init(p.A, p.lda, m0, p.M, p.K, tid);
  lb.init(p.B, p.ldb, n0, p.N, p.K, tid);
  Vec16<bf16_t> ra[2][2], rb[2][2];
  auto fetch = [&](int kt, Vec16<bf16_t>(&a)[2], Vec16<bf16_t>(&b)[2]) {
    if (kt < kt1) {
      la.load(kt, tid, a);
      lb.load(kt, tid, b);
    }
  };
  auto put = [&](int stage, const Vec16<bf16_t>(&a)[2], const Vec16<bf16_t>(&b)[2]) {
    store_lds<TA, PERM>(sA[stage], tid, a);
    store_lds<TB, PERM>(sB[stage], tid, b);
  };
  // pipeline: LDS stage kt&1 holds tile kt; registers hold tile kt+1 (arrived or arriving)
  // and tile kt+2 (just requested)
  fetch(kt0, ra[0], rb[0]);
  if (kt0 < kt1) put(0, ra[0], rb[0]);
  __syncthreads();
  for (int kt = kt0; kt < kt1; ++kt) {
    const int cur = (kt - kt0) & 1;
    fetch(kt + 1, ra[0], rb[0]);
    mma_tile<TA, TB>(sA[cur], sB[cur], arow, brow, lane, acc);
    if (kt + 1 < kt1) put(cur ^ 1, ra[0], rb[0]);
    __syncthreads();
  }

  // accumulator register r of lane l: row 8*(r/4) + 4*(l/32) + r%4, column l%32
  const bool split = gridDim.y > 1;
  int m_base = m0 + wm * 64 + 4 * (lane / 32), n_base = n0 + wn * 64 + lane % 32;
  asm volatile("" : "+v"(m_base), "+v"(n_base));   // keep the output addressing out of the main loop
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int n = n_base + j * 32;
    if (n >= p.N) continue;
    const float bias_v = p.bias ? to_f32(p.bias[n]) : 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m_base + i * 32 + 8 * (r / 4) + r % 4;
        if (m >= p.M) continue;
        const int64_t ci = int64_t(m) * p.ldc + n;
        float v = acc[i][j][r] + bias_v;
        if (p.res)
          v += p.res_fp32 ? reinterpret_cast<const float *>(p.res)[int64_t(m) * p.ldr + n]
                          : to_f32(p.res[int64_t(m) * p.ldr + n]);
        if (split) {
          atomicAdd(static_cast<float *>(p.C) + ci, v);
        } else if (p.c_fp32) {
          float *c = static_cast<float *>(p.C);
          c[ci] = p.accumulate ? c[ci] + v : v;
        } else {
          const bf16_t o = from_f32<bf16_t>(v);
          static_cast<bf16_t *>(p.C)[ci] = o;
          if (p.gelu_out) p.gelu_out[ci] = from_f32<bf16_t>(gelu_f(to_f32(o)));
        }
      }
  }
}

inline int check_launch(const char *what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(HMY_E_HIP, "launch of %s failed: %s", what, hipGetErrorString(e));
  return HMY_OK;
}

}  // namespace

int launch_gemm_mfma32(const hmy_gemm_desc &g, stream_t st) {
  BigP p;
  p.A = static_cast<const bf16_t *>(g.A); p.B = static_cast<const bf16_t *>(g.B); p.C = g.C;
  p.bias = static_cast<const bf16_t *>(g.bias); p.res = static_cast<const bf16_t *>(g.res);
  p.gelu_out = static_cast<bf16_t *>(g.gelu_out);
  p.M = g.M; p.N = g.N; p.K = g.K;
  p.lda = uint32_t(g.lda); p.ldb = uint32_t(g.ldb); p.ldc = g.ldc; p.ldr = g.ldr;
  p.c_fp32 = g.c_fp32; p.accumulate = g.accumulate; p.res_fp32 = g.res_fp32;
  const int gm = (g.M + BM - 1) / BM, gn = (g.N + BM - 1) / BM, nk = (g.K + BK - 1) / BK;
  // split the contraction over workgroups (fp32 atomics into C) when an accumulating
  // GEMM has too few output tiles to fill 256 compute units several times over
  int splits = 1;
  if (g.accumulate && g.c_fp32 && !g.bias && !g.res && gm * gn < 512)
    splits = std::max(1, std::min((768 + gm * gn - 1) / (gm * gn), nk / 8));
  const int tiles_per_split = (nk + splits - 1) / splits;
  splits = (nk + tiles_per_split - 1) / tiles_per_split;
  dim3 grid(gm * gn, splits), block(NT);
  hipStream_t s = (hipStream_t)st;
  if (!g.ta && !g.tb) hipLaunchKernelGGL((k_gemm_mfma32<false, false>), grid, block, 0, s, p, tiles_per_split, gn);
  else if (!g.ta && g.tb) hipLaunchKernelGGL((k_gemm_mfma32<false, true>), grid, block, 0, s, p, tiles_per_split, gn);
  else if (g.ta && !g.tb) hipLaunchKernelGGL((k_gemm_mfma32<true, false>), grid, block, 0, s, p, tiles_per_split, gn);
  else hipLaunchKernelGGL((k_gemm_mfma32<true, true>), grid, block, 0, s, p, tiles_per_split, gn);
  return check_launch("gemm_mfma32");
}

}  // namespace hmy
