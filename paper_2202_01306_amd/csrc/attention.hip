// Softmax attention forward and backward, never materialising the s x s
// probabilities: one thread owns one query row (forward, dQ) or one key row
// (dK, dV); key/value (or query/dO) tiles of 32 rows are staged through LDS and
// read as broadcasts.  Forward keeps the per-row logsumexp; backward recomputes
// probabilities from it.
//
// qkv is [T, 3d] with q | k | v thirds, head h at columns h*DH..; row t belongs to
// sequence t / s, position t % s.
#include "dev_common.h"
#include "hmy_internal.h"

namespace hmy {

namespace {

constexpr int kRows = 64;   // rows (threads) per block
constexpr int kTile = 32;   // staged rows per LDS tile

inline int check_launch(const char *what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(HMY_E_HIP, "launch of %s failed: %s", what, hipGetErrorString(e));
  return HMY_OK;
}

// cooperative copy of `rows` rows x DH columns (row stride ld elements) into LDS [kTile][DH]
template <typename E, int DH>
__device__ __forceinline__ void stage_tile(E *dst, const E *src, int64_t ld, int rows) {
  constexpr int VEC = ElemTraits<E>::VEC;
  constexpr int vec_per_row = DH / VEC;
  for (int i = threadIdx.x; i < kTile * vec_per_row; i += kRows) {
    const int r = i / vec_per_row, c = (i % vec_per_row) * VEC;
    Vec16<E> v;
    if (r < rows) {
      v = load16(src + int64_t(r) * ld + c);
    } else {
#pragma unroll
      for (int k = 0; k < VEC; ++k) v.v[k] = from_f32<E>(0.f);
    }
    store16(dst + r * DH + c, v);
  }
}

template <typename E, int DH>
__device__ __forceinline__ float dot_lds(const float (&q)[DH], const E *row) {
  constexpr int VEC = ElemTraits<E>::VEC;
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < DH; c += VEC) {
    const Vec16<E> v = load16(row + c);
#pragma unroll
    for (int k = 0; k < VEC; ++k) s = fmaf(q[c + k], to_f32(v.v[k]), s);
  }
  return s;
}
template <typename E, int DH>
__device__ __forceinline__ void axpy_lds(float (&acc)[DH], float a, const E *row) {
  constexpr int VEC = ElemTraits<E>::VEC;
#pragma unroll
  for (int c = 0; c < DH; c += VEC) {
    const Vec16<E> v = load16(row + c);
#pragma unroll
    for (int k = 0; k < VEC; ++k) acc[c + k] = fmaf(a, to_f32(v.v[k]), acc[c + k]);
  }
}
template <typename E, int DH>
__device__ __forceinline__ void load_row(float (&dst)[DH], const E *src) {
  constexpr int VEC = ElemTraits<E>::VEC;
#pragma unroll
  for (int c = 0; c < DH; c += VEC) {
    const Vec16<E> v = load16(src + c);
#pragma unroll
    for (int k = 0; k < VEC; ++k) dst[c + k] = to_f32(v.v[k]);
  }
}
template <typename E, int DH>
__device__ __forceinline__ void store_row(E *dst, const float (&src)[DH], float scale) {
  constexpr int VEC = ElemTraits<E>::VEC;
#pragma unroll
  for (int c = 0; c < DH; c += VEC) {
    Vec16<E> v;
#pragma unroll
    for (int k = 0; k < VEC; ++k) v.v[k] = from_f32<E>(src[c + k] * scale);
    store16(dst + c, v);
  }
}

// grid (ceil(s/kRows), H, b), block kRows
template <typename E, int DH>
__global__ __launch_bounds__(kRows) void k_attn_fwd(const E *qkv, E *o, float *lse, int s, int H, int causal) {
  __shared__ __attribute__((aligned(16))) E sK[kTile * DH];
  __shared__ __attribute__((aligned(16))) E sV[kTile * DH];
  const int d = H * DH, ld = 3 * d;
  const int h = blockIdx.y, seq = blockIdx.z;
  const int i0 = blockIdx.x * kRows, i = i0 + threadIdx.x;
  const bool active = i < s;
  const E *base = qkv + int64_t(seq) * s * ld + h * DH;
  const float scale = rsqrtf(float(DH));
  float q[DH], acc[DH];
#pragma unroll
  for (int c = 0; c < DH; ++c) { q[c] = 0.f; acc[c] = 0.f; }
  if (active) load_row<E, DH>(q, base + int64_t(i) * ld);
  float mrun = -INFINITY, lrun = 0.f;
  const int j_end = causal ? min(s, i0 + kRows) : s;   // keys any row of this block may see
  for (int j0 = 0; j0 < j_end; j0 += kTile) {
    const int rows = min(kTile, s - j0);
    __syncthreads();
    stage_tile<E, DH>(sK, base + d + int64_t(j0) * ld, ld, rows);
    stage_tile<E, DH>(sV, base + 2 * d + int64_t(j0) * ld, ld, rows);
    __syncthreads();
    float sc[kTile];
    float tmax = -INFINITY;
#pragma unroll
    for (int jj = 0; jj < kTile; ++jj) {
      const int j = j0 + jj;
      const bool ok = active && jj < rows && (!causal || j <= i);
      sc[jj] = ok ? dot_lds<E, DH>(q, sK + jj * DH) * scale : -INFINITY;
      tmax = fmaxf(tmax, sc[jj]);
    }
    if (tmax == -INFINITY) continue;   // nothing visible in this tile for this row
    const float mnew = fmaxf(mrun, tmax);
    const float corr = __expf(mrun - mnew);   // exp(-inf) = 0 on the first tile
    lrun *= corr;
#pragma unroll
    for (int c = 0; c < DH; ++c) acc[c] *= corr;
#pragma unroll
    for (int jj = 0; jj < kTile; ++jj) {
      if (sc[jj] == -INFINITY) continue;
      const float pj = __expf(sc[jj] - mnew);
      lrun += pj;
      axpy_lds<E, DH>(acc, pj, sV + jj * DH);
    }
    mrun = mnew;
  }
  if (active) {
    store_row<E, DH>(o + (int64_t(seq) * s + i) * d + h * DH, acc, 1.f / lrun);
    lse[(int64_t(seq) * H + h) * s + i] = mrun + __logf(lrun);
  }
}

// delta[seq,h,i] = sum_c do[i,c] * o[i,c]
template <typename E, int DH>
__global__ void k_attn_delta(const E *o, const E *d_o, float *delta, int T, int s, int H) {
  const int64_t idx = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (idx >= int64_t(T) * H) return;
  const int t = int(idx / H), h = int(idx % H);
  const int d = H * DH;
  float a[DH], b[DH];
  load_row<E, DH>(a, o + int64_t(t) * d + h * DH);
  load_row<E, DH>(b, d_o + int64_t(t) * d + h * DH);
  float acc = 0.f;
#pragma unroll
  for (int c = 0; c < DH; ++c) acc = fmaf(a[c], b[c], acc);
  delta[(int64_t(t / s) * H + h) * s + t % s] = acc;
}

// dQ: one thread per query row
template <typename E, int DH>
__global__ __launch_bounds__(kRows) void k_attn_bwd_dq(const E *qkv, const E *d_o, const float *lse, const float *delta,
                                                       E *dqkv, int s, int H, int causal) {
  __shared__ __attribute__((aligned(16))) E sK[kTile * DH];
  __shared__ __attribute__((aligned(16))) E sV[kTile * DH];
  const int d = H * DH, ld = 3 * d;
  const int h = blockIdx.y, seq = blockIdx.z;
  const int i0 = blockIdx.x * kRows, i = i0 + threadIdx.x;
  const bool active = i < s;
  const E *base = qkv + int64_t(seq) * s * ld + h * DH;
  const float scale = rsqrtf(float(DH));
  float q[DH], g[DH], dq[DH];
#pragma unroll
  for (int c = 0; c < DH; ++c) { q[c] = 0.f; g[c] = 0.f; dq[c] = 0.f; }
  float L = 0.f, dl = 0.f;
  if (active) {
    load_row<E, DH>(q, base + int64_t(i) * ld);
    load_row<E, DH>(g, d_o + (int64_t(seq) * s + i) * d + h * DH);
    L = lse[(int64_t(seq) * H + h) * s + i];
    dl = delta[(int64_t(seq) * H + h) * s + i];
  }
  const int j_end = causal ? min(s, i0 + kRows) : s;
  for (int j0 = 0; j0 < j_end; j0 += kTile) {
    const int rows = min(kTile, s - j0);
    __syncthreads();
    stage_tile<E, DH>(sK, base + d + int64_t(j0) * ld, ld, rows);
    stage_tile<E, DH>(sV, base + 2 * d + int64_t(j0) * ld, ld, rows);
    __syncthreads();
    for (int jj = 0; jj < rows; ++jj) {
      const int j = j0 + jj;
      if (!active || (causal && j > i)) continue;
      const float p = __expf(dot_lds<E, DH>(q, sK + jj * DH) * scale - L);
      const float dp = dot_lds<E, DH>(g, sV + jj * DH);
      axpy_lds<E, DH>(dq, p * (dp - dl), sK + jj * DH);
    }
  }
  if (active) store_row<E, DH>(dqkv + (int64_t(seq) * s + i) * ld + h * DH, dq, scale);
}

// dK (PASS 1) or dV (PASS 0): one thread per key row, queries staged through LDS
template <typename E, int DH, int PASS>
__global__ __launch_bounds__(kRows) void k_attn_bwd_dkv(const E *qkv, const E *d_o, const float *lse, const float *delta,
                                                        E *dqkv, int s, int H, int causal) {
  __shared__ __attribute__((aligned(16))) E sQ[kTile * DH];
  __shared__ __attribute__((aligned(16))) E sG[kTile * DH];
  __shared__ float sL[kTile], sD[kTile];
  const int d = H * DH, ld = 3 * d;
  const int h = blockIdx.y, seq = blockIdx.z;
  const int j0 = blockIdx.x * kRows, j = j0 + threadIdx.x;
  const bool active = j < s;
  const E *base = qkv + int64_t(seq) * s * ld + h * DH;
  const float scale = rsqrtf(float(DH));
  float kr[DH], vr[PASS ? DH : 1], acc[DH];
#pragma unroll
  for (int c = 0; c < DH; ++c) { kr[c] = 0.f; acc[c] = 0.f; }
  if (active) {
    load_row<E, DH>(kr, base + d + int64_t(j) * ld);
    if (PASS) load_row<E, DH>(reinterpret_cast<float(&)[DH]>(vr), base + 2 * d + int64_t(j) * ld);
  }
  const int i_begin = causal ? (j0 / kTile) * kTile : 0;   // queries before this block's first key see none of it
  for (int i0 = i_begin; i0 < s; i0 += kTile) {
    const int rows = min(kTile, s - i0);
    __syncthreads();
    stage_tile<E, DH>(sQ, base + int64_t(i0) * ld, ld, rows);
    stage_tile<E, DH>(sG, d_o + (int64_t(seq) * s + i0) * d + h * DH, d, rows);
    if (threadIdx.x < kTile) {
      const bool ok = threadIdx.x < rows;
      sL[threadIdx.x] = ok ? lse[(int64_t(seq) * H + h) * s + i0 + threadIdx.x] : 0.f;
      sD[threadIdx.x] = ok ? delta[(int64_t(seq) * H + h) * s + i0 + threadIdx.x] : 0.f;
    }
    __syncthreads();
    for (int ii = 0; ii < rows; ++ii) {
      const int i = i0 + ii;
      if (!active || (causal && j > i)) continue;
      const float p = __expf(dot_lds<E, DH>(kr, sQ + ii * DH) * scale - sL[ii]);
      if (PASS == 0) {
        axpy_lds<E, DH>(acc, p, sG + ii * DH);                    // dV += P^T dO
      } else {
        const float dp = dot_lds<E, DH>(reinterpret_cast<const float(&)[DH]>(vr), sG + ii * DH);
        axpy_lds<E, DH>(acc, p * (dp - sD[ii]), sQ + ii * DH);    // dK += dS^T Q
      }
    }
  }
  if (active)
    store_row<E, DH>(dqkv + (int64_t(seq) * s + j) * ld + (PASS ? d : 2 * d) + h * DH, acc, PASS ? scale : 1.f);
}

template <typename E, int DH>
int attn_fwd_t(const void *qkv, void *o, float *lse, int b, int s, int H, int causal, hipStream_t st) {
  dim3 grid((s + kRows - 1) / kRows, H, b);
  hipLaunchKernelGGL((k_attn_fwd<E, DH>), grid, dim3(kRows), 0, st, (const E *)qkv, (E *)o, lse, s, H, causal);
  return check_launch("attn_fwd");
}
template <typename E, int DH>
int attn_bwd_t(const void *qkv, const void *o, const void *d_o, const float *lse, float *delta, void *dqkv, int b, int s,
               int H, int causal, hipStream_t st) {
  const int T = b * s;
  const int64_t n = int64_t(T) * H;
  hipLaunchKernelGGL((k_attn_delta<E, DH>), dim3(int((n + 127) / 128)), dim3(128), 0, st, (const E *)o, (const E *)d_o,
                     delta, T, s, H);
  dim3 grid((s + kRows - 1) / kRows, H, b);
  hipLaunchKernelGGL((k_attn_bwd_dq<E, DH>), grid, dim3(kRows), 0, st, (const E *)qkv, (const E *)d_o, lse, delta,
                     (E *)dqkv, s, H, causal);
  hipLaunchKernelGGL((k_attn_bwd_dkv<E, DH, 0>), grid, dim3(kRows), 0, st, (const E *)qkv, (const E *)d_o, lse, delta,
                     (E *)dqkv, s, H, causal);
  hipLaunchKernelGGL((k_attn_bwd_dkv<E, DH, 1>), grid, dim3(kRows), 0, st, (const E *)qkv, (const E *)d_o, lse, delta,
                     (E *)dqkv, s, H, causal);
  return check_launch("attn_bwd");
}

}  // namespace

#define DISPATCH_ATTN(prec, dh, FN, ...)                                          \
  do {                                                                            \
    if ((prec) == HMY_PREC_FP32) {                                                \
      if ((dh) == 32) return FN<float, 32>(__VA_ARGS__);                          \
      if ((dh) == 64) return FN<float, 64>(__VA_ARGS__);                          \
      if ((dh) == 128) return FN<float, 128>(__VA_ARGS__);                        \
    } else if ((prec) == HMY_PREC_BF16) {                                         \
      if ((dh) == 32) return FN<bf16_t, 32>(__VA_ARGS__);                         \
      if ((dh) == 64) return FN<bf16_t, 64>(__VA_ARGS__);                         \
      if ((dh) == 128) return FN<bf16_t, 128>(__VA_ARGS__);                       \
    }                                                                             \
    return fail(HMY_E_INVALID, "attention: unsupported precision %d / head dim %d", prec, dh); \
  } while (0)

int launch_attn_fwd(int prec, const void *qkv, void *o, float *lse, int b, int s, int H, int dh, int causal,
                    stream_t st) {
  if (b < 1 || s < 1 || H < 1) return fail(HMY_E_INVALID, "attn_fwd: bad shape");
  if (prec == HMY_PREC_BF16 && g_use_mfma) return launch_attn_fwd_mfma(qkv, o, lse, b, s, H, dh, causal, st);
  DISPATCH_ATTN(prec, dh, attn_fwd_t, qkv, o, lse, b, s, H, causal, (hipStream_t)st);
}
int launch_attn_bwd(int prec, const void *qkv, const void *o, const void *d_o, const float *lse, float *delta, void *dqkv,
                    float *dbias, int b, int s, int H, int dh, int causal, stream_t st) {
  if (b < 1 || s < 1 || H < 1) return fail(HMY_E_INVALID, "attn_bwd: bad shape");
  if (prec == HMY_PREC_BF16 && g_use_mfma)
    return launch_attn_bwd_mfma(qkv, o, d_o, lse, delta, dqkv, dbias, b, s, H, dh, causal, st);
  // the plain kernels leave the bias gradient to a pass of its own over dqkv
  const int rc = [&]() -> int { DISPATCH_ATTN(prec, dh, attn_bwd_t, qkv, o, d_o, lse, delta, dqkv, b, s, H, causal, (hipStream_t)st); }();
  if (rc != HMY_OK || !dbias) return rc;
  return launch_colsum(prec, dqkv, dbias, b * s, 3 * H * dh, st);
}

}  // namespace hmy
