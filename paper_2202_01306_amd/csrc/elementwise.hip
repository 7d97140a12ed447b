// HBM-bound kernels: embedding, LayerNorm, GELU, bias-gradient column sums,
// softmax cross-entropy, fused Adam, fill and copy.  One wavefront (64 lanes)
// per row for the row reductions; 16-byte accesses along the contiguous axis.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdlib>

#include "dev_common.h"
#include "hmy_internal.h"

namespace hmy {

namespace {

constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / kWave;

inline int grid_for(uint64_t work_items, int per_block, int cap = 1 << 16) {
  uint64_t g = (work_items + per_block - 1) / per_block;
  if (g < 1) g = 1;
  if (g > uint64_t(cap)) g = cap;
  return int(g);
}

inline int check_launch(const char *what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(HMY_E_HIP, "launch of %s failed: %s", what, hipGetErrorString(e));
  return HMY_OK;
}

// ---- fill / copy ---------------------------------------------------------------
__global__ void k_fill_zero(uint32_t *p, uint64_t n_words) {
  const uint64_t stride = uint64_t(gridDim.x) * blockDim.x;
  const uint64_t n4 = n_words / 4;
  uint4 *p4 = reinterpret_cast<uint4 *>(p);
  for (uint64_t i = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n4; i += stride) p4[i] = make_uint4(0, 0, 0, 0);
  for (uint64_t i = n4 * 4 + uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n_words; i += stride) p[i] = 0;
}
__global__ void k_copy(uint32_t *dst, const uint32_t *src, uint64_t n_words) {
  const uint64_t stride = uint64_t(gridDim.x) * blockDim.x;
  const uint64_t n4 = n_words / 4;
  uint4 *d4 = reinterpret_cast<uint4 *>(dst);
  const uint4 *s4 = reinterpret_cast<const uint4 *>(src);
  for (uint64_t i = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n4; i += stride) d4[i] = s4[i];
  for (uint64_t i = n4 * 4 + uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n_words; i += stride) dst[i] = src[i];
}
// HBM -> pinned host memory.  Stores to the host drain at link speed; more of them
// outstanding than the link needs back up into the memory fabric and slow every other
// kernel on the device (measured: a streaming kernel runs 7x slower beside an
// unthrottled 32x256-thread copy, 1.1x beside this one).  So: few, narrow workgroups,
// each waiting for its store before the next.
__global__ void k_copy_out(uint4 *dst, const uint4 *src, uint64_t n4) {
  const uint64_t stride = uint64_t(gridDim.x) * blockDim.x;
  for (uint64_t i = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n4; i += stride) {
    dst[i] = src[i];
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
}

// dst[i] = E(src[i])
template <typename E>
__global__ void k_convert_f32(const float *src, E *dst, uint64_t nvec) {
  constexpr int VEC = ElemTraits<E>::VEC;
  for (uint64_t i = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < nvec; i += uint64_t(gridDim.x) * blockDim.x) {
    Vec16<E> o;
#pragma unroll
    for (int k = 0; k < VEC; ++k) o.v[k] = from_f32<E>(src[i * VEC + k]);
    store16(dst + i * VEC, o);
  }
}

// ---- the residual stream ----------------------------------------------------------
// The activations that run from block to block (x, and their gradients on the way back) are
// fp32 in every precision: each block adds a small update to a large running sum, and rounding
// that sum to bf16 after every addition lets the errors of 2 x n_blocks roundings pile up in
// it (about 1.5 % of its size after 24 blocks, which every gradient then inherits).  Everything
// a block computes from the stream is still the element type E.
template <int VEC> __device__ __forceinline__ void load_stream(const float *p, float (&v)[VEC]) {
#pragma unroll
  for (int k = 0; k < VEC; k += 4) {
    const float4 a = *reinterpret_cast<const float4 *>(p + k);
    v[k] = a.x; v[k + 1] = a.y; v[k + 2] = a.z; v[k + 3] = a.w;
  }
}
template <int VEC> __device__ __forceinline__ void store_stream(float *p, const float (&v)[VEC]) {
#pragma unroll
  for (int k = 0; k < VEC; k += 4) *reinterpret_cast<float4 *>(p + k) = make_float4(v[k], v[k + 1], v[k + 2], v[k + 3]);
}

// dst[i] = float(src[i])
template <typename E>
__global__ void k_convert_to_f32(const E *src, float *dst, uint64_t nvec) {
  constexpr int VEC = ElemTraits<E>::VEC;
  for (uint64_t i = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < nvec; i += uint64_t(gridDim.x) * blockDim.x) {
    const Vec16<E> a = load16(src + i * VEC);
    float v[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) v[k] = to_f32(a.v[k]);
    store_stream<VEC>(dst + i * VEC, v);
  }
}

// ---- embedding ---------------------------------------------------------------
template <typename E>
__global__ void k_embed_fwd(const int32_t *ids, const E *wte, const E *wpe, float *x, int T, int d, int s) {
  constexpr int VEC = ElemTraits<E>::VEC;
  const int vec_per_row = d / VEC;
  const uint64_t total = uint64_t(T) * vec_per_row;
  for (uint64_t i = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += uint64_t(gridDim.x) * blockDim.x) {
    const int t = int(i / vec_per_row), c = int(i % vec_per_row) * VEC;
    const Vec16<E> a = load16(wte + uint64_t(ids[t]) * d + c);
    const Vec16<E> p = load16(wpe + uint64_t(t % s) * d + c);
    float o[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) o[k] = to_f32(a.v[k]) + to_f32(p.v[k]);
    store_stream<VEC>(x + uint64_t(t) * d + c, o);
  }
}
// dwte[id[t]] += dx[t]  (rows may repeat: atomics)
__global__ void k_embed_bwd_wte(const int32_t *ids, const float *dx, float *dwte, int T, int d) {
  constexpr int VEC = 4;
  const int vec_per_row = d / VEC;
  const uint64_t total = uint64_t(T) * vec_per_row;
  for (uint64_t i = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += uint64_t(gridDim.x) * blockDim.x) {
    const int t = int(i / vec_per_row), c = int(i % vec_per_row) * VEC;
    float g[VEC];
    load_stream<VEC>(dx + uint64_t(t) * d + c, g);
    float *dst = dwte + uint64_t(ids[t]) * d + c;
#pragma unroll
    for (int k = 0; k < VEC; ++k) atomicAdd(dst + k, g[k]);
  }
}
// dwpe[j] += sum over sequences of dx[i*s + j]  (one owner per element: no atomics)
__global__ void k_embed_bwd_wpe(const float *dx, float *dwpe, int T, int d, int s) {
  constexpr int VEC = 4;
  const int vec_per_row = d / VEC;
  const int nseq = T / s;
  const uint64_t total = uint64_t(s) * vec_per_row;
  for (uint64_t i = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += uint64_t(gridDim.x) * blockDim.x) {
    const int j = int(i / vec_per_row), c = int(i % vec_per_row) * VEC;
    float acc[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) acc[k] = 0.f;
    for (int q = 0; q < nseq; ++q) {
      float g[VEC];
      load_stream<VEC>(dx + (uint64_t(q) * s + j) * d + c, g);
#pragma unroll
      for (int k = 0; k < VEC; ++k) acc[k] += g[k];
    }
    float *dst = dwpe + uint64_t(j) * d + c;
#pragma unroll
    for (int k = 0; k < VEC; ++k) dst[k] += acc[k];
  }
}

// ---- LayerNorm -----------------------------------------------------------------
// One wavefront per row.  Mean, then biased variance about the mean, then the
// normalised output; the row is re-read from cache between passes.  x is the fp32
// residual stream; gamma, beta and the output have the element type.
template <typename E>
__global__ void k_layernorm_fwd(const float *x, const E *gamma, const E *beta, E *y, float *mean, float *rstd, int T, int d,
                                float eps) {
  constexpr int VEC = ElemTraits<E>::VEC;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  for (int row = blockIdx.x * kWavesPerBlock + wave; row < T; row += gridDim.x * kWavesPerBlock) {
    const float *xr = x + uint64_t(row) * d;
    float s = 0.f;
    for (int c = lane * VEC; c < d; c += kWave * VEC) {
      float v[VEC];
      load_stream<VEC>(xr + c, v);
#pragma unroll
      for (int k = 0; k < VEC; ++k) s += v[k];
    }
    const float mu = wave_sum(s) / float(d);
    float q = 0.f;
    for (int c = lane * VEC; c < d; c += kWave * VEC) {
      float v[VEC];
      load_stream<VEC>(xr + c, v);
#pragma unroll
      for (int k = 0; k < VEC; ++k) {
        const float t = v[k] - mu;
        q += t * t;
      }
    }
    const float rs = rsqrtf(wave_sum(q) / float(d) + eps);
    if (lane == 0) {
      mean[row] = mu;
      rstd[row] = rs;
    }
    E *yr = y + uint64_t(row) * d;
    for (int c = lane * VEC; c < d; c += kWave * VEC) {
      float v[VEC];
      load_stream<VEC>(xr + c, v);
      const Vec16<E> g = load16(gamma + c), b = load16(beta + c);
      Vec16<E> o;
#pragma unroll
      for (int k = 0; k < VEC; ++k) o.v[k] = from_f32<E>(to_f32(g.v[k]) * ((v[k] - mu) * rs) + to_f32(b.v[k]));
      store16(yr + c, o);
    }
  }
}

// The same for rows of at most 64 * VEC * NJ elements, with the row kept in registers: one
// trip to memory instead of three dependent ones (the kernel is a single wave of rows at the
// sizes it runs at, so its time is latency, not bandwidth).  Same arithmetic: mean, then
// biased variance about the mean.
template <typename E, int NJ>
__global__ __launch_bounds__(kBlock) void k_layernorm_fwd_reg(const float *x, const E *gamma, const E *beta, E *y, float *mean, float *rstd, int T,
                                    int d, float eps) {
  constexpr int VEC = ElemTraits<E>::VEC;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  Vec16<E> gm[NJ], bt[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int c = VEC * (lane + kWave * j);
    if (c < d) {
      gm[j] = load16(gamma + c);
      bt[j] = load16(beta + c);
    }
  }
  for (int row = blockIdx.x * kWavesPerBlock + wave; row < T; row += gridDim.x * kWavesPerBlock) {
    const float *xr = x + uint64_t(row) * d;
    float xv[NJ][VEC];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int c = VEC * (lane + kWave * j);
      if (c < d) load_stream<VEC>(xr + c, xv[j]);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      if (VEC * (lane + kWave * j) < d) {
#pragma unroll
        for (int k = 0; k < VEC; ++k) s += xv[j][k];
      }
    }
    const float mu = wave_sum(s) / float(d);
    float q = 0.f;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      if (VEC * (lane + kWave * j) < d) {
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
          const float t = xv[j][k] - mu;
          q += t * t;
        }
      }
    }
    const float rs = rsqrtf(wave_sum(q) / float(d) + eps);
    if (lane == 0) {
      mean[row] = mu;
      rstd[row] = rs;
    }
    E *yr = y + uint64_t(row) * d;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int c = VEC * (lane + kWave * j);
      if (c < d) {
        Vec16<E> o;
#pragma unroll
        for (int k = 0; k < VEC; ++k)
          o.v[k] = from_f32<E>(to_f32(gm[j].v[k]) * ((xv[j][k] - mu) * rs) + to_f32(bt[j].v[k]));
        store16(yr + c, o);
      }
    }
  }
}

// dx = res + (dxhat - mean(dxhat) - xhat*mean(dxhat*xhat)) * rstd, dxhat = dy*gamma;
// dgamma += sum_rows dy*xhat, dbeta += sum_rows dy.  x, res and dx are the fp32 residual stream;
// dx_e, if given, receives dx rounded to the element type (the copy that feeds the GEMMs).
// Per-block partial column sums live in LDS (2*d floats) and are flushed with one atomic per column.
template <typename E>
__global__ void k_layernorm_bwd(const E *dy, const float *x, const float *mean, const float *rstd, const E *gamma,
                                const float *res, float *dx, E *dx_e, float *dgamma, float *dbeta, int T, int d) {
  constexpr int VEC = ElemTraits<E>::VEC;
  extern __shared__ float lds[];
  float *s_dg = lds, *s_db = lds + d;
  for (int c = threadIdx.x; c < 2 * d; c += blockDim.x) lds[c] = 0.f;
  __syncthreads();
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  for (int row = blockIdx.x * kWavesPerBlock + wave; row < T; row += gridDim.x * kWavesPerBlock) {
    const float *xr = x + uint64_t(row) * d;
    const E *dyr = dy + uint64_t(row) * d;
    const float mu = mean[row], rs = rstd[row];
    float s1 = 0.f, s2 = 0.f;
    for (int c = lane * VEC; c < d; c += kWave * VEC) {
      float xv[VEC];
      load_stream<VEC>(xr + c, xv);
      const Vec16<E> gv = load16(dyr + c), gm = load16(gamma + c);
#pragma unroll
      for (int k = 0; k < VEC; ++k) {
        const float xh = (xv[k] - mu) * rs;
        const float g = to_f32(gv.v[k]);
        const float dxh = g * to_f32(gm.v[k]);
        s1 += dxh;
        s2 += dxh * xh;
        atomicAdd(&s_dg[c + k], g * xh);
        atomicAdd(&s_db[c + k], g);
      }
    }
    s1 = wave_sum(s1) / float(d);
    s2 = wave_sum(s2) / float(d);
    float *dxr = dx + uint64_t(row) * d;
    const float *rr = res ? res + uint64_t(row) * d : nullptr;
    for (int c = lane * VEC; c < d; c += kWave * VEC) {
      float xv[VEC], rv[VEC], o[VEC];
      load_stream<VEC>(xr + c, xv);
      const Vec16<E> gv = load16(dyr + c), gm = load16(gamma + c);
      if (rr) load_stream<VEC>(rr + c, rv);
      Vec16<E> oe;
#pragma unroll
      for (int k = 0; k < VEC; ++k) {
        const float xh = (xv[k] - mu) * rs;
        const float dxh = to_f32(gv.v[k]) * to_f32(gm.v[k]);
        float v = (dxh - s1 - xh * s2) * rs;
        if (rr) v += rv[k];
        o[k] = v;
        oe.v[k] = from_f32<E>(v);
      }
      store_stream<VEC>(dxr + c, o);
      if (dx_e) store16(dx_e + uint64_t(row) * d + c, oe);
    }
  }
  __syncthreads();
  for (int c = threadIdx.x; c < d; c += blockDim.x) {
    atomicAdd(&dgamma[c], s_dg[c]);
    atomicAdd(&dbeta[c], s_db[c]);
  }
}

// ---- GELU ------------------------------------------------------------------------
template <typename E>
__global__ void k_gelu_fwd(const E *u, E *g, uint64_t nvec) {
  constexpr int VEC = ElemTraits<E>::VEC;
  for (uint64_t i = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < nvec; i += uint64_t(gridDim.x) * blockDim.x) {
    const Vec16<E> a = load16(u + i * VEC);
    Vec16<E> o;
#pragma unroll
    for (int k = 0; k < VEC; ++k) o.v[k] = from_f32<E>(gelu_f(to_f32(a.v[k])));
    store16(g + i * VEC, o);
  }
}
template <typename E>
__global__ void k_gelu_bwd(const E *dg, const E *u, E *du, uint64_t nvec) {
  constexpr int VEC = ElemTraits<E>::VEC;
  for (uint64_t i = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < nvec; i += uint64_t(gridDim.x) * blockDim.x) {
    const Vec16<E> a = load16(u + i * VEC), b = load16(dg + i * VEC);
    Vec16<E> o;
#pragma unroll
    for (int k = 0; k < VEC; ++k) o.v[k] = from_f32<E>(to_f32(b.v[k]) * gelu_grad_f(to_f32(a.v[k])));
    store16(du + i * VEC, o);
  }
}

// The same with the column sums of du (the gradient of the bias in front of the activation) added into
// `db`: grid and reduction of k_colsum, so that du is not read again by a kernel of its own.  The sums are
// taken over du as stored (rounded to E), which is what that kernel would have read.
template <typename E>
__global__ void k_gelu_bwd_colsum(const E *dg, const E *u, E *du, float *db, int T, int N, int rows_per_split) {
  constexpr int VEC = ElemTraits<E>::VEC;
  __shared__ float part[kWavesPerBlock][kWave * VEC];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int c = (blockIdx.x * kWave + lane) * VEC;
  const int r0 = blockIdx.y * rows_per_split, r1 = min(T, r0 + rows_per_split);
  float acc[VEC];
#pragma unroll
  for (int k = 0; k < VEC; ++k) acc[k] = 0.f;
  if (c < N) {
    auto one = [&](const Vec16<E> &a, const Vec16<E> &b, int r) {
      Vec16<E> o;
#pragma unroll
      for (int k = 0; k < VEC; ++k) {
        o.v[k] = from_f32<E>(to_f32(b.v[k]) * gelu_grad_f(to_f32(a.v[k])));
        acc[k] += to_f32(o.v[k]);
      }
      store16(du + uint64_t(r) * N + c, o);
    };
    int r = r0 + wave;
    for (; r + kWavesPerBlock < r1; r += 2 * kWavesPerBlock) {   // two rows in flight
      const uint64_t i0 = uint64_t(r) * N + c, i1 = uint64_t(r + kWavesPerBlock) * N + c;
      const Vec16<E> a0 = load16(u + i0), b0 = load16(dg + i0), a1 = load16(u + i1), b1 = load16(dg + i1);
      one(a0, b0, r);
      one(a1, b1, r + kWavesPerBlock);
    }
    for (; r < r1; r += kWavesPerBlock) {
      const uint64_t i0 = uint64_t(r) * N + c;
      one(load16(u + i0), load16(dg + i0), r);
    }
  }
#pragma unroll
  for (int k = 0; k < VEC; ++k) part[wave][lane * VEC + k] = acc[k];
  __syncthreads();
  for (int i = threadIdx.x; i < kWave * VEC; i += blockDim.x) {
    const int col = blockIdx.x * kWave * VEC + i;
    if (col < N) {
      float t = 0.f;
#pragma unroll
      for (int w = 0; w < kWavesPerBlock; ++w) t += part[w][i];
      atomicAdd(db + col, t);
    }
  }
}

// LayerNorm backward for rows of at most 64 * VEC * NJ elements: lane l owns columns
// VEC * (l + 64 j) .. + VEC - 1, j < NJ, and keeps their dgamma / dbeta partial sums in
// registers over all the rows its wave visits; one pass over x and dy (kept in
// registers between the two phases).  Each wave then writes its sums to its own row of
// LDS, the workgroup adds the rows up, and one row per workgroup goes to the workspace
// (or, without one, into dgamma / dbeta with atomics).  With `dres` the column sums of `res` are
// taken along in the same way (ns = 3 sums per column instead of 2): `res` is the gradient that arrives
// over the residual connection, i.e. the gradient of the output of the linear layer that closes the
// branch, and its column sums are the gradient of that layer's bias.
template <typename E, int NJ>
// one workgroup of 16 / 8 / 4 waves per compute unit (its LDS rows allow no more), i.e. 4 / 2 / 1 waves per
// SIMD: the bounds tell the compiler that it may use 128 / 256 / 512 registers; left to itself it aimed at 64
// and spilled the row to scratch memory
__global__ __launch_bounds__(NJ <= 1 ? 1024 : NJ <= 4 ? 512 : 256)
    __attribute__((amdgpu_waves_per_eu(1, NJ <= 1 ? 4 : NJ <= 4 ? 2 : 1))) void k_layernorm_bwd_reg(const E *dy, const float *x, const float *mean, const float *rstd,
                                                          const E *gamma, const float *res, float *dx, E *dx_e, float *dgamma, float *dbeta,
                                                          float *dres, int T, int d, float *partial) {
  constexpr int VEC = ElemTraits<E>::VEC;
  extern __shared__ __align__(16) float lds[];   // per wave: dgamma[d], dbeta[d] (, dres[d])
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave, waves = blockDim.x / kWave;
  const bool sum_res = dres != nullptr;
  const int ns = sum_res ? 3 : 2;
  float dg[NJ][VEC], db[NJ][VEC], dr[NJ][VEC];
  Vec16<E> gm[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int c = VEC * (lane + kWave * j);
    if (c < d) gm[j] = load16(gamma + c);
#pragma unroll
    for (int k = 0; k < VEC; ++k) dg[j][k] = db[j][k] = dr[j][k] = 0.f;
  }
  for (int row = blockIdx.x * waves + wave; row < T; row += gridDim.x * waves) {
    const float *xr = x + uint64_t(row) * d;
    const E *dyr = dy + uint64_t(row) * d;
    const float mu = mean[row], rs = rstd[row];
    float xv[NJ][VEC];
    Vec16<E> gv[NJ];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int c = VEC * (lane + kWave * j);
      if (c < d) {
        load_stream<VEC>(xr + c, xv[j]);
        gv[j] = load16(dyr + c);
      }
    }
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int c = VEC * (lane + kWave * j);
      if (c < d) {
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
          const float xh = (xv[j][k] - mu) * rs;
          xv[j][k] = xh;   // only the normalised value is needed from here on
          const float g = to_f32(gv[j].v[k]);
          const float dxh = g * to_f32(gm[j].v[k]);
          s1 += dxh;
          s2 += dxh * xh;
          dg[j][k] += g * xh;
          db[j][k] += g;
        }
      }
    }
    s1 = wave_sum(s1) / float(d);
    s2 = wave_sum(s2) / float(d);
    float *dxr = dx + uint64_t(row) * d;
    const float *rr = res ? res + uint64_t(row) * d : nullptr;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int c = VEC * (lane + kWave * j);
      if (c < d) {
        float rv[VEC], o[VEC];
        if (rr) load_stream<VEC>(rr + c, rv);
        Vec16<E> oe;
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
          const float dxh = to_f32(gv[j].v[k]) * to_f32(gm[j].v[k]);
          float v = (dxh - s1 - xv[j][k] * s2) * rs;
          if (rr) v += rv[k];
          if (sum_res) dr[j][k] += rv[k];
          o[k] = v;
          oe.v[k] = from_f32<E>(v);
        }
        store_stream<VEC>(dxr + c, o);
        if (dx_e) store16(dx_e + uint64_t(row) * d + c, oe);
      }
    }
  }
  float *mine = lds + uint64_t(wave) * ns * d;
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int c = VEC * (lane + kWave * j);
    if (c < d) {
      // 16-byte stores: scalar ones from lanes VEC floats apart would pile onto a few LDS banks
#pragma unroll
      for (int k = 0; k < VEC; k += 4) {
        *reinterpret_cast<float4 *>(mine + c + k) = make_float4(dg[j][k], dg[j][k + 1], dg[j][k + 2], dg[j][k + 3]);
        *reinterpret_cast<float4 *>(mine + d + c + k) = make_float4(db[j][k], db[j][k + 1], db[j][k + 2], db[j][k + 3]);
        if (sum_res)
          *reinterpret_cast<float4 *>(mine + 2 * d + c + k) = make_float4(dr[j][k], dr[j][k + 1], dr[j][k + 2], dr[j][k + 3]);
      }
    }
  }
  __syncthreads();
  float *row = partial ? partial + uint64_t(blockIdx.x) * ns * d : nullptr;
  for (int c = threadIdx.x; c < ns * d; c += blockDim.x) {
    float t = 0.f;
    for (int w = 0; w < waves; ++w) t += lds[uint64_t(w) * ns * d + c];
    if (row) row[c] = t;   // one row of sums per workgroup; k_ln_bwd_reduce adds them up
    else atomicAdd(c < d ? &dgamma[c] : c < 2 * d ? &dbeta[c - d] : &dres[c - 2 * d], t);
  }
}

// The same for wider rows: WPR waves share a row, each owning a band of 2 * 64 * VEC columns (two 16-byte
// vectors per lane, as in the register kernel's best case), so that a row of 1600 or 4096 columns neither spills
// nor leaves one wave per SIMD.  A workgroup of 8 waves works on 8 / WPR rows at a time; the two row sums meet in
// LDS (one barrier per row, two alternating buffers), added in the same order by every wave of the row.  Every
// wave runs the same number of rounds (rows past the end are skipped inside the round), so the barriers match.
template <typename E, int WPR>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(1, 2))) void k_layernorm_bwd_wide(
    const E *dy, const float *x, const float *mean, const float *rstd, const E *gamma, const float *res, float *dx, E *dx_e,
    float *dgamma, float *dbeta, float *dres, int T, int d, float *partial) {
  constexpr int VEC = ElemTraits<E>::VEC, NJ = 2, kWaves = 8, kSlots = kWaves / WPR, kBand = NJ * kWave * VEC;
  extern __shared__ __align__(16) float lds[];   // per row slot: dgamma[d], dbeta[d] (, dres[d]); then the row sums' exchange
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int slot = wave / WPR, col0 = (wave % WPR) * kBand;
  const bool sum_res = dres != nullptr;
  const int ns = sum_res ? 3 : 2;
  float *xch = lds + uint64_t(kSlots) * ns * d;   // [2][kWaves][2]
  float dg[NJ][VEC], db[NJ][VEC], dr[NJ][VEC];
  Vec16<E> gm[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int c = col0 + VEC * (lane + kWave * j);
    if (c < d) gm[j] = load16(gamma + c);
#pragma unroll
    for (int k = 0; k < VEC; ++k) dg[j][k] = db[j][k] = dr[j][k] = 0.f;
  }
  int round = 0;
  for (int base = blockIdx.x * kSlots; base < T; base += gridDim.x * kSlots, ++round) {
    const int row = base + slot;
    const bool live = row < T;
    const float *xr = x + uint64_t(live ? row : 0) * d;
    const E *dyr = dy + uint64_t(live ? row : 0) * d;
    const float mu = live ? mean[row] : 0.f, rs = live ? rstd[row] : 0.f;
    float xv[NJ][VEC];
    Vec16<E> gv[NJ];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int c = col0 + VEC * (lane + kWave * j);
      if (live && c < d) {
        load_stream<VEC>(xr + c, xv[j]);
        gv[j] = load16(dyr + c);
      }
    }
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int c = col0 + VEC * (lane + kWave * j);
      if (live && c < d) {
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
          const float xh = (xv[j][k] - mu) * rs;
          xv[j][k] = xh;
          const float g = to_f32(gv[j].v[k]);
          const float dxh = g * to_f32(gm[j].v[k]);
          s1 += dxh;
          s2 += dxh * xh;
          dg[j][k] += g * xh;
          db[j][k] += g;
        }
      }
    }
    s1 = wave_sum(s1);
    s2 = wave_sum(s2);
    float *mine = xch + (round & 1) * (2 * kWaves);
    if (lane == 0) {
      mine[2 * wave] = s1;
      mine[2 * wave + 1] = s2;
    }
    __syncthreads();
    s1 = s2 = 0.f;
#pragma unroll
    for (int w = 0; w < WPR; ++w) {
      s1 += mine[2 * (slot * WPR + w)];
      s2 += mine[2 * (slot * WPR + w) + 1];
    }
    s1 /= float(d);
    s2 /= float(d);
    if (live) {
      float *dxr = dx + uint64_t(row) * d;
      const float *rr = res ? res + uint64_t(row) * d : nullptr;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const int c = col0 + VEC * (lane + kWave * j);
        if (c < d) {
          float rv[VEC], o[VEC];
          if (rr) load_stream<VEC>(rr + c, rv);
          Vec16<E> oe;
#pragma unroll
          for (int k = 0; k < VEC; ++k) {
            const float dxh = to_f32(gv[j].v[k]) * to_f32(gm[j].v[k]);
            float v = (dxh - s1 - xv[j][k] * s2) * rs;
            if (rr) v += rv[k];
            if (sum_res) dr[j][k] += rv[k];
            o[k] = v;
            oe.v[k] = from_f32<E>(v);
          }
          store_stream<VEC>(dxr + c, o);
          if (dx_e) store16(dx_e + uint64_t(row) * d + c, oe);
        }
      }
    }
  }
  // the waves of a row slot hold disjoint bands of columns: together they fill the slot's row of sums
  float *mine = lds + uint64_t(slot) * ns * d;
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int c = col0 + VEC * (lane + kWave * j);
    if (c < d) {
#pragma unroll
      for (int k = 0; k < VEC; k += 4) {
        *reinterpret_cast<float4 *>(mine + c + k) = make_float4(dg[j][k], dg[j][k + 1], dg[j][k + 2], dg[j][k + 3]);
        *reinterpret_cast<float4 *>(mine + d + c + k) = make_float4(db[j][k], db[j][k + 1], db[j][k + 2], db[j][k + 3]);
        if (sum_res)
          *reinterpret_cast<float4 *>(mine + 2 * d + c + k) = make_float4(dr[j][k], dr[j][k + 1], dr[j][k + 2], dr[j][k + 3]);
      }
    }
  }
  __syncthreads();
  float *out_row = partial ? partial + uint64_t(blockIdx.x) * ns * d : nullptr;
  for (int c = threadIdx.x; c < ns * d; c += blockDim.x) {
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < kSlots; ++w) t += lds[uint64_t(w) * ns * d + c];
    if (out_row) out_row[c] = t;
    else atomicAdd(c < d ? &dgamma[c] : c < 2 * d ? &dbeta[c - d] : &dres[c - 2 * d], t);
  }
}

// dgamma += column sums of partial[:, 0:d], dbeta += those of partial[:, d:2d] and, with rows of 3 d sums,
// dres += those of partial[:, 2d:3d].  The launches that accumulate into one tensor are ordered on their
// stream, so plain adds do.
__global__ void k_ln_bwd_reduce(const float *partial, int rows, int d, int ns, float *dgamma, float *dbeta, float *dres) {
  __shared__ float part[4][64];
  const int tx = threadIdx.x % 64, ty = threadIdx.x / 64;   // 64 columns x 4 interleaved row groups
  const int c = blockIdx.x * 64 + tx;
  const int w = ns * d;   // floats per row of partial sums
  float t = 0.f;
  if (c < w) {
    int r = ty;
    for (; r + 28 < rows; r += 32) {
      float v[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) v[q] = partial[uint64_t(r + 4 * q) * w + c];
#pragma unroll
      for (int q = 0; q < 8; ++q) t += v[q];
    }
    for (; r < rows; r += 4) t += partial[uint64_t(r) * w + c];
  }
  part[ty][tx] = t;
  __syncthreads();
  if (ty == 0 && c < w) {
    t = part[0][tx] + part[1][tx] + part[2][tx] + part[3][tx];
    if (c < d) dgamma[c] += t;
    else if (c < 2 * d) dbeta[c - d] += t;
    else dres[c - 2 * d] += t;
  }
}

// ---- column sums (bias gradients) ---------------------------------------------
// grid = (column groups of 64*VEC, row splits).  A wave reads whole 64*VEC-column row
// segments (16 bytes per lane), four rows in flight; the workgroup's waves take
// interleaved rows, combine through LDS, and one atomic per column leaves the workgroup.
template <typename E>
__global__ void k_colsum(const E *a, float *out, int T, int N, int rows_per_split) {
  constexpr int VEC = ElemTraits<E>::VEC;
  __shared__ float part[kWavesPerBlock][kWave * VEC];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int c = (blockIdx.x * kWave + lane) * VEC;
  const int r0 = blockIdx.y * rows_per_split, r1 = min(T, r0 + rows_per_split);
  float acc[VEC];
#pragma unroll
  for (int k = 0; k < VEC; ++k) acc[k] = 0.f;
  if (c < N) {
    int r = r0 + wave;
    for (; r + 3 * kWavesPerBlock < r1; r += 4 * kWavesPerBlock) {
      Vec16<E> v[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) v[q] = load16(a + uint64_t(r + q * kWavesPerBlock) * N + c);
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc[k] += to_f32(v[q].v[k]);
    }
    for (; r < r1; r += kWavesPerBlock) {
      const Vec16<E> v = load16(a + uint64_t(r) * N + c);
#pragma unroll
      for (int k = 0; k < VEC; ++k) acc[k] += to_f32(v.v[k]);
    }
  }
#pragma unroll
  for (int k = 0; k < VEC; ++k) part[wave][lane * VEC + k] = acc[k];
  __syncthreads();
  for (int i = threadIdx.x; i < kWave * VEC; i += blockDim.x) {
    const int col = blockIdx.x * kWave * VEC + i;
    if (col < N) {
      float t = 0.f;
#pragma unroll
      for (int w = 0; w < kWavesPerBlock; ++w) t += part[w][i];
      atomicAdd(out + col, t);
    }
  }
}

// ---- softmax cross-entropy ---------------------------------------------------
__device__ __forceinline__ float block_reduce(float v, bool is_max, float *scratch) {
  v = is_max ? wave_max(v) : wave_sum(v);
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  __syncthreads();
  if (lane == 0) scratch[wave] = v;
  __syncthreads();
  float r = scratch[0];
  for (int w = 1; w < kWavesPerBlock; ++w) r = is_max ? fmaxf(r, scratch[w]) : r + scratch[w];
  return r;
}

// One workgroup per row.  Pass 1 keeps a running (max, sum of exponentials) pair per
// thread over 16-byte loads and merges the pairs across the workgroup; pass 2 re-reads
// the row (it is still in L2) and writes the gradient, 8 columns per thread per step.
template <typename E>
__global__ void k_xent(const float *logits, const int32_t *targets, double *loss_acc, E *dlogits, int V, int64_t ldl,
                       float inv_ntgt) {
  __shared__ float scratch[kWavesPerBlock];
  const int row = blockIdx.x;
  const float *lr = logits + uint64_t(row) * ldl;
  E *dr = dlogits + uint64_t(row) * ldl;
  const int tgt = targets[row];
  const bool vec = (ldl % 8 == 0) && ((reinterpret_cast<uintptr_t>(logits) & 15) == 0) &&
                   ((reinterpret_cast<uintptr_t>(dlogits) & 15) == 0) && sizeof(E) == 2;
  const int nv = vec ? int(ldl / 8) : 0;   // 8-column groups handled with vector accesses
  if (tgt < 0) {
    Vec16<E> z;
#pragma unroll
    for (int k = 0; k < ElemTraits<E>::VEC; ++k) z.v[k] = from_f32<E>(0.f);
    for (int j = threadIdx.x; j < nv; j += blockDim.x) store16(dr + 8 * j, z);
    for (int j = nv * 8 + threadIdx.x; j < ldl; j += blockDim.x) dr[j] = from_f32<E>(0.f);
    return;
  }
  float mx = -INFINITY, se = 0.f;
  auto take = [&](float v) {
    if (v > mx) {
      se = se * __expf(mx - v) + 1.f;
      mx = v;
    } else {
      se += __expf(v - mx);
    }
  };
  for (int j = threadIdx.x; j < nv; j += blockDim.x) {
    float v[8];
    *reinterpret_cast<float4 *>(v) = *reinterpret_cast<const float4 *>(lr + 8 * j);
    *reinterpret_cast<float4 *>(v + 4) = *reinterpret_cast<const float4 *>(lr + 8 * j + 4);
#pragma unroll
    for (int k = 0; k < 8; ++k)
      if (8 * j + k < V) take(v[k]);
  }
  for (int j = nv * 8 + threadIdx.x; j < V; j += blockDim.x) take(lr[j]);
  const float gmx = block_reduce(mx, true, scratch);
  se = mx == -INFINITY ? 0.f : se * __expf(mx - gmx);
  se = block_reduce(se, false, scratch);
  const float lse = gmx + logf(se);
  if (threadIdx.x == 0) atomicAdd(loss_acc, double(lse - lr[tgt]) * double(inv_ntgt));
  for (int j = threadIdx.x; j < nv; j += blockDim.x) {
    float v[8];
    *reinterpret_cast<float4 *>(v) = *reinterpret_cast<const float4 *>(lr + 8 * j);
    *reinterpret_cast<float4 *>(v + 4) = *reinterpret_cast<const float4 *>(lr + 8 * j + 4);
    Vec16<E> o;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int col = 8 * j + k;
      const float g = col < V ? (__expf(v[k] - lse) - (col == tgt ? 1.f : 0.f)) * inv_ntgt : 0.f;
      if (k < ElemTraits<E>::VEC) o.v[k] = from_f32<E>(g);
    }
    store16(dr + 8 * j, o);
  }
  for (int j = nv * 8 + threadIdx.x; j < ldl; j += blockDim.x) {
    float g = 0.f;
    if (j < V) g = (__expf(lr[j] - lse) - (j == tgt ? 1.f : 0.f)) * inv_ntgt;
    dr[j] = from_f32<E>(g);
  }
}

// ---- fused Adam ---------------------------------------------------------------
// mixed: fp32 master/m/v in, updated master/m/v + RNE-rounded compute weight out.
// fp32:  the fp32 weight is the master (W == float, master == w_out).
template <typename W>
__global__ void k_adam(const float *grad, float *master, float *m, float *v, W *w_out, uint64_t n, float lr, float b1,
                       float b2, float eps, float inv_bc1, float inv_bc2) {
  const uint64_t stride = uint64_t(gridDim.x) * blockDim.x;
  const uint64_t n4 = n / 4;
  for (uint64_t i = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n4 + (n % 4 ? 1 : 0); i += stride) {
    const uint64_t base = i * 4;
    const int cnt = int(min<uint64_t>(4, n - base));
    for (int k = 0; k < cnt; ++k) {
      const uint64_t j = base + k;
      const float g = grad[j];
      const float mm = b1 * m[j] + (1.f - b1) * g;
      const float vv = b2 * v[j] + (1.f - b2) * g * g;
      const float w = master[j] - lr * (mm * inv_bc1) / (sqrtf(vv * inv_bc2) + eps);
      m[j] = mm;
      v[j] = vv;
      master[j] = w;
      if (sizeof(W) == 2) w_out[j] = from_f32<W>(w);
    }
  }
}

// Fused Adam + swap-out: reads the gradient from HBM and the optimizer state from
// wherever in_* point (the HBM ring), and writes the updated state, the compute-
// precision weight and the gradient straight to the caller's pinned host arrays
// (out_*: host pointers, written over the host link as full 16/32-byte vectors).
// MIXED: master/m/v fp32 + bf16 weight.  !MIXED: the fp32 weight is the master
// (in_master = the weight in HBM, out_w is fp32 and out_master is not used).
// out_g == nullptr: the gradient is not exported.  Eight elements per thread per step; n may have a tail.
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
// 16 bytes to pinned host memory as a streaming store (nothing of it needs to stay in the L2 on the way out)
__device__ __forceinline__ void store_host4(float *dst, const float *src) {
  __builtin_nontemporal_store(*reinterpret_cast<const f32x4 *>(src), reinterpret_cast<f32x4 *>(dst));
}

// At most 64 registers: the kernel runs beside the compute stream's, and the largest of those leave 64 registers per
// lane of a compute unit they occupy -- with more, a unit that holds one wave of this kernel could not take their workgroup.
template <bool MIXED>
__global__ __attribute__((amdgpu_waves_per_eu(8))) void k_adam_out(const float *grad, const float *in_master, const float *in_m, const float *in_v,
                           float *out_master, float *out_m, float *out_v, void *out_w, float *out_g, uint64_t n,
                           float lr, float b1, float b2, float eps, float inv_bc1, float inv_bc2) {
  // A wavefront takes 512 consecutive elements per step as two runs of 256: lane l holds elements
  // 4 l .. 4 l + 3 of each run, so that every store instruction writes one contiguous KiB (half a KiB for the
  // bf16 weight).  With eight consecutive elements per lane each instruction left 16-byte holes between
  // lanes, which the path to the host has to stitch together from two instructions.
  // The wave's position is kept in scalar registers (it is the same for all lanes), so that every access is a
  // uniform base plus a lane offset of 32 bits: per-lane 64-bit addresses for nine arrays would cost the registers
  // that the cap above takes away.
  const int lane = threadIdx.x % kWave;
  const uint64_t wave = uint64_t(__builtin_amdgcn_readfirstlane(int((blockIdx.x * blockDim.x + threadIdx.x) / kWave)));
  const uint64_t stride = uint64_t(gridDim.x) * blockDim.x * 8;
  for (uint64_t wb = wave * 512; wb < n; wb += stride) {
    float g[8], w[8], m[8], v[8];
    uint64_t at[2];
    bool full[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      at[h] = wb + 256 * h + 4 * lane;
      full[h] = at[h] + 4 <= n;
      if (full[h]) {
        *reinterpret_cast<float4 *>(g + 4 * h) = *reinterpret_cast<const float4 *>(grad + at[h]);
        *reinterpret_cast<float4 *>(w + 4 * h) = *reinterpret_cast<const float4 *>(in_master + at[h]);
        *reinterpret_cast<float4 *>(m + 4 * h) = *reinterpret_cast<const float4 *>(in_m + at[h]);
        *reinterpret_cast<float4 *>(v + 4 * h) = *reinterpret_cast<const float4 *>(in_v + at[h]);
      } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const bool ok = at[h] + k < n;
          g[4 * h + k] = ok ? grad[at[h] + k] : 0.f;
          w[4 * h + k] = ok ? in_master[at[h] + k] : 0.f;
          m[4 * h + k] = ok ? in_m[at[h] + k] : 0.f;
          v[4 * h + k] = ok ? in_v[at[h] + k] : 0.f;
        }
      }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      m[k] = b1 * m[k] + (1.f - b1) * g[k];
      v[k] = b2 * v[k] + (1.f - b2) * g[k] * g[k];
      w[k] = w[k] - lr * (m[k] * inv_bc1) / (sqrtf(v[k] * inv_bc2) + eps);
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      if (full[h]) {
        store_host4(out_m + at[h], m + 4 * h);
        store_host4(out_v + at[h], v + 4 * h);
        if (out_g) store_host4(out_g + at[h], g + 4 * h);
        if (MIXED) {
          store_host4(out_master + at[h], w + 4 * h);
          bf16_t o[4];
#pragma unroll
          for (int k = 0; k < 4; ++k) o[k] = from_f32<bf16_t>(w[4 * h + k]);
          __builtin_nontemporal_store(*reinterpret_cast<const u32x2 *>(o), reinterpret_cast<u32x2 *>(static_cast<bf16_t *>(out_w) + at[h]));
        } else {
          store_host4(static_cast<float *>(out_w) + at[h], w + 4 * h);
        }
      } else {
        for (int k = 0; k < 4 && at[h] + k < n; ++k) {
          const uint64_t j = at[h] + k;
          out_m[j] = m[4 * h + k];
          out_v[j] = v[4 * h + k];
          if (out_g) out_g[j] = g[4 * h + k];
          if (MIXED) {
            out_master[j] = w[4 * h + k];
            static_cast<bf16_t *>(out_w)[j] = from_f32<bf16_t>(w[4 * h + k]);
          } else {
            static_cast<float *>(out_w)[j] = w[4 * h + k];
          }
        }
      }
    }
    // bound the stores to the host that are outstanding (see k_copy_out)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
}

}  // namespace

#define DISPATCH_PREC(prec, CALL)                                 \
  do {                                                              \
    if ((prec) == HMY_PREC_FP32) { typedef float E; CALL; }         \
    else if ((prec) == HMY_PREC_BF16) { typedef bf16_t E; CALL; }   \
    else return fail(HMY_E_INVALID, "unknown precision %d", prec);  \
  } while (0)

int launch_fill_zero(void *p, uint64_t bytes, stream_t st) {
  if (!bytes) return HMY_OK;
  if (bytes % 4 || (reinterpret_cast<uintptr_t>(p) & 15)) return fail(HMY_E_INVALID, "fill_zero: unaligned");
  const uint64_t words = bytes / 4;
  hipLaunchKernelGGL(k_fill_zero, dim3(grid_for(words / 4 + 1, kBlock, 2048)), dim3(kBlock), 0, (hipStream_t)st,
                     (uint32_t *)p, words);
  return check_launch("fill_zero");
}
int launch_copy(void *dst, const void *src, uint64_t bytes, stream_t st, int grid_cap) {
  if (!bytes) return HMY_OK;
  if (bytes % 4 || (reinterpret_cast<uintptr_t>(dst) & 15) || (reinterpret_cast<uintptr_t>(src) & 15))
    return fail(HMY_E_INVALID, "copy: unaligned");
  const uint64_t words = bytes / 4;
  hipLaunchKernelGGL(k_copy, dim3(grid_for(words / 4 + 1, kBlock, grid_cap)), dim3(kBlock), 0, (hipStream_t)st,
                     (uint32_t *)dst, (const uint32_t *)src, words);
  return check_launch("copy");
}

int launch_copy_out(void *dst_host, const void *src, uint64_t bytes, stream_t st) {
  if (!bytes) return HMY_OK;
  if (bytes % 16 || (reinterpret_cast<uintptr_t>(dst_host) & 15) || (reinterpret_cast<uintptr_t>(src) & 15))
    return fail(HMY_E_INVALID, "copy_out: unaligned");
  hipLaunchKernelGGL(k_copy_out, dim3(32), dim3(64), 0, (hipStream_t)st, (uint4 *)dst_host, (const uint4 *)src, bytes / 16);
  return check_launch("copy_out");
}

int launch_convert_f32(int prec, const float *src, void *dst, uint64_t n, stream_t st) {
  if (n % 8) return fail(HMY_E_INVALID, "convert: n must be a multiple of 8");
  DISPATCH_PREC(prec, {
    const uint64_t nvec = n / ElemTraits<E>::VEC;
    hipLaunchKernelGGL(k_convert_f32<E>, dim3(grid_for(nvec, kBlock, 4096)), dim3(kBlock), 0, (hipStream_t)st, src,
                       (E *)dst, nvec);
  });
  return check_launch("convert_f32");
}

int launch_embed_fwd(int prec, const int32_t *ids, const void *wte, const void *wpe, float *x, int T, int d, int s,
                     int vocab, stream_t st) {
  (void)vocab;
  if (T < 1 || d % 8 || s < 1) return fail(HMY_E_INVALID, "embed_fwd: bad shape");
  DISPATCH_PREC(prec, {
    const uint64_t work = uint64_t(T) * (d / ElemTraits<E>::VEC);
    hipLaunchKernelGGL(k_embed_fwd<E>, dim3(grid_for(work, kBlock, 4096)), dim3(kBlock), 0, (hipStream_t)st, ids,
                       (const E *)wte, (const E *)wpe, x, T, d, s);
  });
  return check_launch("embed_fwd");
}
int launch_embed_bwd(int prec, const int32_t *ids, const float *dx, float *dwte, float *dwpe, int T, int d, int s,
                     int vocab, stream_t st) {
  (void)vocab;
  if (prec != HMY_PREC_FP32 && prec != HMY_PREC_BF16) return fail(HMY_E_INVALID, "unknown precision %d", prec);
  if (T < 1 || d % 8 || s < 1 || T % s) return fail(HMY_E_INVALID, "embed_bwd: bad shape");
  const uint64_t work = uint64_t(T) * (d / 4);
  hipLaunchKernelGGL(k_embed_bwd_wte, dim3(grid_for(work, kBlock, 4096)), dim3(kBlock), 0, (hipStream_t)st, ids, dx, dwte, T,
                     d);
  const uint64_t work2 = uint64_t(s) * (d / 4);
  hipLaunchKernelGGL(k_embed_bwd_wpe, dim3(grid_for(work2, kBlock, 4096)), dim3(kBlock), 0, (hipStream_t)st, dx, dwpe, T, d, s);
  return check_launch("embed_bwd");
}
int launch_convert_to_f32(int prec, const void *src, float *dst, uint64_t n, stream_t st) {
  if (n % 8) return fail(HMY_E_INVALID, "convert: n must be a multiple of 8");
  DISPATCH_PREC(prec, {
    const uint64_t nvec = n / ElemTraits<E>::VEC;
    hipLaunchKernelGGL(k_convert_to_f32<E>, dim3(grid_for(nvec, kBlock, 4096)), dim3(kBlock), 0, (hipStream_t)st,
                       (const E *)src, dst, nvec);
  });
  return check_launch("convert_to_f32");
}

template <typename E>
void launch_ln_fwd(const float *x, const E *gamma, const E *beta, E *y, float *mean, float *rstd, int T, int d, float eps,
                   hipStream_t st) {
  const int nj = (d + kWave * ElemTraits<E>::VEC - 1) / (kWave * ElemTraits<E>::VEC);
  const dim3 g(grid_for(T, kWavesPerBlock, 8192)), b(kBlock);
  if (nj == 1) hipLaunchKernelGGL((k_layernorm_fwd_reg<E, 1>), g, b, 0, st, x, gamma, beta, y, mean, rstd, T, d, eps);
  else if (nj == 2) hipLaunchKernelGGL((k_layernorm_fwd_reg<E, 2>), g, b, 0, st, x, gamma, beta, y, mean, rstd, T, d, eps);
  else if (nj <= 4) hipLaunchKernelGGL((k_layernorm_fwd_reg<E, 4>), g, b, 0, st, x, gamma, beta, y, mean, rstd, T, d, eps);
  else if (nj <= 8) hipLaunchKernelGGL((k_layernorm_fwd_reg<E, 8>), g, b, 0, st, x, gamma, beta, y, mean, rstd, T, d, eps);
  else hipLaunchKernelGGL(k_layernorm_fwd<E>, g, b, 0, st, x, gamma, beta, y, mean, rstd, T, d, eps);
}

int launch_layernorm_fwd(int prec, const float *x, const void *gamma, const void *beta, void *y, float *mean, float *rstd,
                         int T, int d, float eps, stream_t st) {
  if (T < 1 || d % 8) return fail(HMY_E_INVALID, "layernorm_fwd: bad shape");
  DISPATCH_PREC(prec, launch_ln_fwd<E>(x, (const E *)gamma, (const E *)beta, (E *)y, mean, rstd, T, d, eps, (hipStream_t)st));
  return check_launch("layernorm_fwd");
}
template <typename E>
void launch_ln_bwd(const E *dy, const float *x, const float *mean, const float *rstd, const E *gamma, const float *res,
                   float *dx, E *dx_e, float *dgamma, float *dbeta, float *dres, int T, int d, hipStream_t st, float *ws,
                   uint64_t ws_bytes) {
  constexpr int VEC = ElemTraits<E>::VEC;
  const int nj = (d + kWave * VEC - 1) / (kWave * VEC);
  const int ns = dres ? 3 : 2;   // sums per column
  if (nj > 2 && nj <= 16) {
    // rows wider than two vectors per lane: several waves per row (2 up to four vectors, 4 up to eight, 8 beyond)
    const int wpr = nj <= 4 ? 2 : nj <= 8 ? 4 : 8, slots = 8 / wpr;
    const int grid = grid_for(T, slots, kLnBlocks);
    float *partial = ws && ws_bytes >= uint64_t(grid) * ns * d * 4 ? ws : nullptr;
    const size_t lds = (size_t(slots) * ns * d + 2 * 8 * 2) * 4;
    const dim3 g(grid), b(8 * kWave);
    if (wpr == 2) hipLaunchKernelGGL((k_layernorm_bwd_wide<E, 2>), g, b, lds, st, dy, x, mean, rstd, gamma, res, dx, dx_e, dgamma, dbeta, dres, T, d, partial);
    else if (wpr == 4) hipLaunchKernelGGL((k_layernorm_bwd_wide<E, 4>), g, b, lds, st, dy, x, mean, rstd, gamma, res, dx, dx_e, dgamma, dbeta, dres, T, d, partial);
    else hipLaunchKernelGGL((k_layernorm_bwd_wide<E, 8>), g, b, lds, st, dy, x, mean, rstd, gamma, res, dx, dx_e, dgamma, dbeta, dres, T, d, partial);
    if (partial)
      hipLaunchKernelGGL(k_ln_bwd_reduce, dim3((ns * d + 63) / 64), dim3(256), 0, st, partial, grid, d, ns, dgamma, dbeta, dres);
    return;
  }
  // waves per workgroup: as many as 128 KiB of LDS holds rows of 2 d floats, and as the registers allow
  // without spilling (16 for rows of one 16-byte vector per lane, 8 up to four vectors, 4 beyond; measured
  // at d = 1024 bf16: 16 waves with spills 22 us, 8 waves 15 us, 4 waves 20 us)
  int waves = 16;
  while (waves > 1 && (uint64_t(waves) * ns * d * 4 > (128u << 10) || (nj > 1 && waves > 8) || (nj > 4 && waves > 4)))
    waves /= 2;   // also the kernels' launch bounds
  const int grid = grid_for(T, waves, kLnBlocks);
  float *partial = ws && ws_bytes >= uint64_t(grid) * ns * d * 4 && nj <= 8 ? ws : nullptr;
  const size_t lds = size_t(waves) * ns * d * 4;
  const dim3 g(grid), b(waves * kWave);
  if (nj == 1) hipLaunchKernelGGL((k_layernorm_bwd_reg<E, 1>), g, b, lds, st, dy, x, mean, rstd, gamma, res, dx, dx_e, dgamma, dbeta, dres, T, d, partial);
  else if (nj == 2) hipLaunchKernelGGL((k_layernorm_bwd_reg<E, 2>), g, b, lds, st, dy, x, mean, rstd, gamma, res, dx, dx_e, dgamma, dbeta, dres, T, d, partial);
  else if (nj <= 4) hipLaunchKernelGGL((k_layernorm_bwd_reg<E, 4>), g, b, lds, st, dy, x, mean, rstd, gamma, res, dx, dx_e, dgamma, dbeta, dres, T, d, partial);
  else if (nj <= 8) hipLaunchKernelGGL((k_layernorm_bwd_reg<E, 8>), g, b, lds, st, dy, x, mean, rstd, gamma, res, dx, dx_e, dgamma, dbeta, dres, T, d, partial);
  else
    hipLaunchKernelGGL(k_layernorm_bwd<E>, dim3(grid_for(T, kWavesPerBlock, 512)), dim3(kBlock), size_t(2) * d * 4, st, dy, x, mean,
                       rstd, gamma, res, dx, dx_e, dgamma, dbeta, T, d);
  if (partial)
    hipLaunchKernelGGL(k_ln_bwd_reduce, dim3((ns * d + 63) / 64), dim3(256), 0, st, partial, grid, d, ns, dgamma, dbeta, dres);
}

int launch_layernorm_bwd(int prec, const void *dy, const float *x, const float *mean, const float *rstd, const void *gamma,
                         const float *res, float *dx, void *dx_e, float *dgamma, float *dbeta, float *dres_sum, int T,
                         int d, stream_t st, float *workspace, uint64_t workspace_bytes) {
  if (T < 1 || d % 8 || d > 8192) return fail(HMY_E_INVALID, "layernorm_bwd: bad shape");
  if (dres_sum && !res) return fail(HMY_E_INVALID, "layernorm_bwd: column sums of a residual gradient that is not given");
  DISPATCH_PREC(prec, {
    if (dres_sum && d > 16 * kWave * ElemTraits<E>::VEC) {
      // rows too wide for the register kernel: the sums get a pass of their own, before dx (which may be res) is written
      const int rc = launch_colsum(HMY_PREC_FP32, res, dres_sum, T, d, st);
      if (rc != HMY_OK) return rc;
      dres_sum = nullptr;
    }
    launch_ln_bwd<E>((const E *)dy, x, mean, rstd, (const E *)gamma, res, dx, (E *)dx_e, dgamma, dbeta, dres_sum, T, d,
                     (hipStream_t)st, workspace, workspace_bytes);
  });
  return check_launch("layernorm_bwd");
}

// ---- LayerNorm backward for callers that cannot allocate -----------------------------
// The partial-sum rows of k_layernorm_bwd_reg live in a file-scope device array instead of a
// caller's workspace.  Every GPU the library runs on holds its own copy of the array at its own
// address; in host code the array's name is only a handle for hipGetSymbolAddress, so the address
// is looked up once per device (with that device current) and kept.
constexpr int kStaticLnMaxD = 4096;   // widest row the static workspace serves
constexpr int kMaxDevices = 64;
__device__ __align__(256) float g_ln_bwd_scratch[uint64_t(kLnBlocks) * 2 * kStaticLnMaxD];   // 8 MiB
namespace {
std::atomic<float *> g_ln_bwd_scratch_ptr[kMaxDevices];

// device address of the scratch array on the current device (nullptr + error recorded on failure)
float *ln_bwd_scratch_on_current_device() {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    fail(HMY_E_HIP, "layernorm_bwd_static: no current device (%s)", hipGetErrorString(e));
    return nullptr;
  }
  float *p = g_ln_bwd_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p) return p;
  void *addr = nullptr;
  e = hipGetSymbolAddress(&addr, HIP_SYMBOL(g_ln_bwd_scratch));
  if (e != hipSuccess || !addr) {
    fail(HMY_E_HIP, "layernorm_bwd_static: hipGetSymbolAddress failed: %s", hipGetErrorString(e));
    return nullptr;
  }
  // two threads racing here look up the same address: either store is right
  g_ln_bwd_scratch_ptr[dev].store(static_cast<float *>(addr), std::memory_order_release);
  return static_cast<float *>(addr);
}
}  // namespace

int launch_layernorm_bwd_static(int prec, const void *dy, const float *x, const float *mean, const float *rstd,
                                const void *gamma, const float *res, float *dx, void *dx_e, float *dgamma, float *dbeta,
                                int T, int d, stream_t st) {
  if (T < 1 || d < 8 || d % 8) return fail(HMY_E_INVALID, "layernorm_bwd_static: bad shape");
  if (d > kStaticLnMaxD)
    return fail(HMY_E_INVALID, "layernorm_bwd_static: d = %d exceeds the static workspace's limit of %d columns; "
                               "use hmy_k_layernorm_bwd with a workspace of the caller's", d, kStaticLnMaxD);
  float *ws = ln_bwd_scratch_on_current_device();
  if (!ws) return HMY_E_HIP;
  // nothing in the workspace has to start at zero: every workgroup overwrites its whole row before
  // the reduction kernel, ordered behind it on the stream, reads the rows of this launch only
  return launch_layernorm_bwd(prec, dy, x, mean, rstd, gamma, res, dx, dx_e, dgamma, dbeta, nullptr, T, d, st, ws,
                              uint64_t(kLnBlocks) * 2 * d * 4);
}

int launch_gelu_fwd(int prec, const void *u, void *g, uint64_t n, stream_t st) {
  if (n % 8) return fail(HMY_E_INVALID, "gelu: n must be a multiple of 8");
  DISPATCH_PREC(prec, {
    const uint64_t nvec = n / ElemTraits<E>::VEC;
    hipLaunchKernelGGL(k_gelu_fwd<E>, dim3(grid_for(nvec, kBlock, 8192)), dim3(kBlock), 0, (hipStream_t)st,
                       (const E *)u, (E *)g, nvec);
  });
  return check_launch("gelu_fwd");
}
int launch_gelu_bwd(int prec, const void *dg, const void *u, void *du, uint64_t n, stream_t st) {
  if (n % 8) return fail(HMY_E_INVALID, "gelu: n must be a multiple of 8");
  DISPATCH_PREC(prec, {
    const uint64_t nvec = n / ElemTraits<E>::VEC;
    hipLaunchKernelGGL(k_gelu_bwd<E>, dim3(grid_for(nvec, kBlock, 8192)), dim3(kBlock), 0, (hipStream_t)st,
                       (const E *)dg, (const E *)u, (E *)du, nvec);
  });
  return check_launch("gelu_bwd");
}

int launch_gelu_bwd_colsum(int prec, const void *dg, const void *u, void *du, float *db, int T, int N, stream_t st) {
  if (T < 1 || N % 8) return fail(HMY_E_INVALID, "gelu_bwd_colsum: bad shape");
  DISPATCH_PREC(prec, {
    const int cols_per_block = kWave * ElemTraits<E>::VEC;
    const int gx = (N + cols_per_block - 1) / cols_per_block;
    int splits = std::max(1, std::min(T / 16, 2048 / gx));
    const int rows_per_split = (T + splits - 1) / splits;
    splits = (T + rows_per_split - 1) / rows_per_split;
    hipLaunchKernelGGL(k_gelu_bwd_colsum<E>, dim3(gx, splits), dim3(kBlock), 0, (hipStream_t)st, (const E *)dg,
                       (const E *)u, (E *)du, db, T, N, rows_per_split);
  });
  return check_launch("gelu_bwd_colsum");
}

int launch_colsum(int prec, const void *a, float *out, int T, int N, stream_t st) {
  if (T < 1 || N % 8) return fail(HMY_E_INVALID, "colsum: bad shape");
  DISPATCH_PREC(prec, {
    const int cols_per_block = kWave * ElemTraits<E>::VEC;
    const int gx = (N + cols_per_block - 1) / cols_per_block;
    int splits = std::max(1, std::min(T / 64, 2048 / gx));
    const int rows_per_split = (T + splits - 1) / splits;
    splits = (T + rows_per_split - 1) / rows_per_split;
    hipLaunchKernelGGL(k_colsum<E>, dim3(gx, splits), dim3(kBlock), 0, (hipStream_t)st, (const E *)a, out, T, N,
                       rows_per_split);
  });
  return check_launch("colsum");
}

int launch_xent(int prec, const float *logits, const int32_t *targets, double *loss_acc, void *dlogits, int T, int V,
                int64_t ldl, float inv_ntgt, stream_t st) {
  if (T < 1 || V < 2 || ldl < V) return fail(HMY_E_INVALID, "xent: bad shape");
  DISPATCH_PREC(prec, {
    hipLaunchKernelGGL(k_xent<E>, dim3(T), dim3(kBlock), 0, (hipStream_t)st, logits, targets, loss_acc, (E *)dlogits, V,
                       ldl, inv_ntgt);
  });
  return check_launch("xent");
}

int launch_adam(int prec, const float *grad, float *master, float *m, float *v, void *w_out, uint64_t n,
                const hmy_adam &hp, stream_t st) {
  if (!n) return HMY_OK;
  if (hp.step < 1) return fail(HMY_E_INVALID, "adam: step is 1-based");
  const float inv_bc1 = float(1.0 / (1.0 - std::pow(double(hp.beta1), double(hp.step))));
  const float inv_bc2 = float(1.0 / (1.0 - std::pow(double(hp.beta2), double(hp.step))));
  const int grid = grid_for(n / 4 + 1, kBlock, 4096);
  if (prec == HMY_PREC_BF16) {
    if (!master) return fail(HMY_E_INVALID, "adam(bf16): master required");
    hipLaunchKernelGGL(k_adam<bf16_t>, dim3(grid), dim3(kBlock), 0, (hipStream_t)st, grad, master, m, v,
                       (bf16_t *)w_out, n, hp.lr, hp.beta1, hp.beta2, hp.eps, inv_bc1, inv_bc2);
  } else if (prec == HMY_PREC_FP32) {
    if (master) return fail(HMY_E_INVALID, "adam(fp32): master must be NULL");
    hipLaunchKernelGGL(k_adam<float>, dim3(grid), dim3(kBlock), 0, (hipStream_t)st, grad, (float *)w_out, m, v,
                       (float *)w_out, n, hp.lr, hp.beta1, hp.beta2, hp.eps, inv_bc1, inv_bc2);
  } else {
    return fail(HMY_E_INVALID, "unknown precision %d", prec);
  }
  return check_launch("adam");
}

int launch_adam_out(int prec, const float *grad, const float *in_master, const float *in_m, const float *in_v,
                    float *out_master, float *out_m, float *out_v, void *out_w, float *out_g, uint64_t n,
                    const hmy_adam &hp, bool alone, stream_t st) {
  if (!n) return HMY_OK;
  if (hp.step < 1) return fail(HMY_E_INVALID, "adam: step is 1-based");
  const float inv_bc1 = float(1.0 / (1.0 - std::pow(double(hp.beta1), double(hp.step))));
  const float inv_bc2 = float(1.0 / (1.0 - std::pow(double(hp.beta2), double(hp.step))));
  // beside the compute stream: narrow workgroups, few of them -- what keeps the link busy
  // without flooding the fabric (see k_copy_out); with the device to itself: enough to
  // run the link at full speed
  static const int cap_env = std::getenv("HMY_ADAM_GRID") ? std::max(1, std::atoi(std::getenv("HMY_ADAM_GRID"))) : 10;
  const int blk = alone ? 256 : 64;
  const int grid = grid_for(n / 8 + 1, blk, alone ? 32 : cap_env);
  if (prec == HMY_PREC_BF16)
    hipLaunchKernelGGL(k_adam_out<true>, dim3(grid), dim3(blk), 0, (hipStream_t)st, grad, in_master, in_m, in_v,
                       out_master, out_m, out_v, out_w, out_g, n, hp.lr, hp.beta1, hp.beta2, hp.eps, inv_bc1, inv_bc2);
  else if (prec == HMY_PREC_FP32)
    hipLaunchKernelGGL(k_adam_out<false>, dim3(grid), dim3(blk), 0, (hipStream_t)st, grad, in_master, in_m, in_v,
                       out_master, out_m, out_v, out_w, out_g, n, hp.lr, hp.beta1, hp.beta2, hp.eps, inv_bc1, inv_bc2);
  else
    return fail(HMY_E_INVALID, "unknown precision %d", prec);
  return check_launch("adam_out");
}

}  // namespace hmy
