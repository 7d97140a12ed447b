// bf16 GEMM on the matrix cores with operand tiles streamed HBM -> LDS by the
// load-to-LDS instruction (global_load_lds_dwordx4): no staging registers, so a ring
// of S LDS stages keeps up to S-1 K tiles in flight per workgroup while one is
// multiplied, which is what hides HBM latency when an operand is not cache-resident
// (activations of another microbatch, weights that have just arrived from the host).
//
// 128x128 block tile, four wavefronts of 64x64 (2x2 v_mfma_f32_32x32x16_bf16), K tile
// BK in {32, 64}.  One s_waitcnt vmcnt + one barrier per K tile, placed inside the tile
// so that the first fragments of the next tile are requested before this tile's last
// multiplies.  Fragments are read one (BK 32) or two (BK 64) 16-deep steps ahead of
// their multiplies; every LDS read and load-to-LDS is issued right behind a multiply.
//
// A load-to-LDS instruction writes 64 lanes x 16 bytes to one contiguous KiB of LDS
// (lane i at byte 16 i) from per-lane global addresses, so the bank swizzle is applied
// on the global side: the lane that owns LDS slot p of a row fetches the chunk that
// the swizzle maps to p.
//
// LDS layouts.  Operand with the contraction index contiguous in memory: [row][k],
// 16-byte chunks XOR-swizzled by the row, read with ds_read_b128.  Operand stored
// contraction-major: kept as loaded, [k][row], chunks swizzled by k, read through
// ds_read_b64_tr_b16 with k rows 8h..8h+3 and 8h+4..8h+7 (h = lane/32), which is the
// same contraction order as the 16-byte read of the other layout.
//
// Tuning switches (read once per process): HMY_GEMM_BK = 32 | 64 overrides the K tile of
// both kernels, HMY_GEMM_STAGES = 3 | 4 the ring depth of the 128x128 kernel,
// HMY_GEMM_TILE = 128 | 256 the choice between it and the 256x256 kernel.
#include <algorithm>
#include <cstdlib>

#include "dev_common.h"
#include "hmy_internal.h"

namespace hmy {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128, NT = 256;  // square block tile, threads

struct DmaP {
  const bf16_t *A, *B;
  void *C;
  const bf16_t *bias, *res;
  bf16_t *gelu_out;
  int M, N, K;
  uint32_t lda, ldb;
  int64_t ldc, ldr;
  int c_fp32, accumulate, res_fp32;
};

// element address inside a [row][k] tile of BK columns (BK/8 chunks per row)
template <int BK>
__device__ __forceinline__ int addr_rk(int row, int chunk) {
  if (BK == 32) return row * 32 + ((chunk ^ ((row >> 2) & 3)) << 3);
  return row * 64 + ((chunk ^ ((row >> 1) & 7)) << 3);
}
// element address inside a [k][row] tile (16 chunks per k-row, swizzled by k)
__device__ __forceinline__ int addr_kr(int k, int col) {
  return k * BM + ((((col >> 3) ^ ((k & 3) << 2)) & 15) << 3) + (col & 7);
}

// one wavefront-wide 16-byte-per-lane copy HBM -> LDS.  lds_addr is wave-uniform (the
// hardware adds 16 * lane); the global address is base + byte offset per lane.
// The statement overwrites m0 and cannot say so: the compiler rejects m0 in a clobber list as a
// reserved register ("may lead to undefined behaviour").  That is safe here because the compiler
// keeps no value of its own in m0 across statements: whenever code it generates reads m0 (indexed
// register moves, messages, its own LDS-direct loads) it writes m0 immediately before, and this
// file uses none of those constructs.
__device__ __forceinline__ void dma16(const void *base, uint32_t byte_off, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(byte_off), "s"(base), "s"(lds_addr)
               : "memory");
}

// Per-thread, loop-invariant byte offsets of this thread's lanes of every KiB it copies.
// TR = false: memory [row][k]; KiB c holds rows c*R..c*R+R-1 (R = 512/BK), lane i owns slot i%(BK/8) of row i/(BK/8).
// TR = true : memory [k][row]; KiB c holds k rows 4c..4c+3, lane i owns slot i%16 of k row i/16.
// Wave w copies KiBs c = 4 j + w, j = 0..BK/16-1.  Rows outside the operand are
// clamped into it: they only feed outputs that are never stored.
template <bool TR, int BK>
struct Dma {
  static constexpr int NJ = BK / 16;
  uint32_t off[TR ? 1 : NJ];
  uint32_t step;  // TR: bytes between this thread's consecutive KiBs
  __device__ __forceinline__ void init(uint32_t ld, int row0, int nrows, int lane, int wave) {
    if (!TR) {
      constexpr int CH = BK / 8, R = 64 / CH;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const int row = (4 * j + wave) * R + lane / CH, slot = lane % CH;
        const int chunk = BK == 32 ? (slot ^ ((row >> 2) & 3)) : (slot ^ ((row >> 1) & 7));
        off[j] = (uint32_t(min(row0 + row, nrows - 1)) * ld + uint32_t(chunk * 8)) * 2u;
      }
      step = 0;
    } else {
      const int kq = lane / 16, slot = lane % 16;
      const int chunk = slot ^ (kq << 2);   // k & 3 == lane / 16 for every KiB
      const int col = min(row0 + chunk * 8, ((nrows + 7) & ~7) - 8);
      off[0] = (uint32_t(4 * wave + kq) * ld + uint32_t(col)) * 2u;
      step = 16u * ld * 2u;
    }
  }
  // base: operand base advanced to the K tile; lds: byte address of the tile's stage
  __device__ __forceinline__ void issue_one(const bf16_t *base, uint32_t lds, int wave, int j) const {
    dma16(base, TR ? off[0] + uint32_t(j) * step : off[j], lds + uint32_t(4 * j + wave) * 1024u);
  }
  __device__ __forceinline__ void issue(const bf16_t *base, uint32_t lds, int wave) const {
#pragma unroll
    for (int j = 0; j < NJ; ++j) issue_one(base, lds, wave, j);
  }
};

template <bool TR, int BK>
__device__ __forceinline__ bf16x8 frag(const bf16_t *s, int row32, int ks, int lane) {
  if (!TR) {
    return *reinterpret_cast<const bf16x8 *>(s + addr_rk<BK>(row32 + lane % 32, 2 * ks + lane / 32));
  } else {
    const int q = lane % 16, g16 = (lane / 16) % 2, h = lane / 32;
    const int k = 16 * ks + 8 * h + q / 4, col = row32 + 16 * g16 + 4 * (q % 4);
    typedef __attribute__((address_space(3))) short4v *lds_ptr;
    union { short4v s4[2]; bf16x8 b; } u;
    u.s4[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(s + addr_kr(k, col)));
    u.s4[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(s + addr_kr(k + 4, col)));
    return u.b;
  }
}

template <int N> __device__ __forceinline__ void wait_vm() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

// Output stage for 8 consecutive columns of one row.  `fast`: every pointer and leading
// dimension allows 16-byte accesses; `inside`: the workgroup's tile lies inside C.  A
// tile that sticks out still leaves through the 16-byte path wherever a row's group of
// 8 columns lies inside C (a 1600-wide output ends in the middle of a tile: element by
// element that tile took longer than the whole K loop); what remains, and everything
// when `fast` is false, goes element by element through a loop kept rolled, so that it
// costs no instruction-cache space.
struct Epi {
  bool fast, inside;
  __device__ __forceinline__ bool whole8(const DmaP &p, int m, int nn) const {
    return inside || (m < p.M && nn + 8 <= p.N);
  }
  __device__ __forceinline__ void init(const DmaP &p, int m0, int n0, int side = BM) {
    const int esz = p.c_fp32 ? 4 : 2;
    bool ok = (reinterpret_cast<uintptr_t>(p.C) & 15) == 0 && (p.ldc * esz) % 16 == 0;
    if (p.res) ok = ok && (reinterpret_cast<uintptr_t>(p.res) & 15) == 0 && p.ldr % 8 == 0;
    if (p.res && p.res_fp32 && p.accumulate) ok = false;   // both would want the prefetch registers
    if (p.bias) ok = ok && (reinterpret_cast<uintptr_t>(p.bias) & 15) == 0;
    if (p.gelu_out) ok = ok && (reinterpret_cast<uintptr_t>(p.gelu_out) & 15) == 0;
    fast = ok;
    inside = m0 + side <= p.M && n0 + side <= p.N;
  }
  // tanh-form GELU with the hardware exponential: the argument is a bf16 value and so is
  // the result, which the 2-ulp exponential does not disturb.  Written as u * sigmoid(2z),
  // the same function as u/2 (1 + tanh z), z = c (u + a u^3), in fewer instructions: the
  // epilogue's arithmetic runs with the matrix cores idle, so it is paid in full.
  static __device__ __forceinline__ float gelu_fast(float u) {
    // exp(-2z) as one exp2 with the constants folded, and the hardware reciprocal: __fdividef and
    // __expf expand to a ten-instruction IEEE division and an extra multiply
    const float k = -2.f * 0.7978845608028654f * 1.4426950408889634f, a = 0.044715f;
    return u * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(k * (u + a * u * u * u)));
  }
  // what the output stage reads from global memory for 8 columns of one row: the residual
  // (bf16) or, for an accumulating fp32 C, C itself.  Fetched before the last K tile so
  // that its latency hides behind that tile's multiplies.
  struct Pre { float4 lo, hi; };
  __device__ __forceinline__ void prefetch(const DmaP &p, int m, int nn, Pre &r) const {
    if (!whole8(p, m, nn)) return;
    if (p.res && p.res_fp32) {   // the fp32 residual stream: 8 columns are 32 bytes
      const float *x = reinterpret_cast<const float *>(p.res) + int64_t(m) * p.ldr + nn;
      r.lo = *reinterpret_cast<const float4 *>(x);
      r.hi = *reinterpret_cast<const float4 *>(x + 4);
    } else if (p.res) {
      r.lo = *reinterpret_cast<const float4 *>(p.res + int64_t(m) * p.ldr + nn);
    } else if (p.c_fp32 && p.accumulate) {
      const float *c = static_cast<const float *>(p.C) + int64_t(m) * p.ldc + nn;
      r.lo = *reinterpret_cast<const float4 *>(c);
      r.hi = *reinterpret_cast<const float4 *>(c + 4);
    }
  }
  // v[0..7] += the eight bf16 values held in the 16 bytes of `raw`, taken apart with integer operations on
  // the registers: reading them through a pointer of another type made the compiler keep `raw` in scratch memory
  static __device__ __forceinline__ void add_bf16x8(float (&v)[8], const float4 &raw) {
    const uint32_t u[4] = {__float_as_uint(raw.x), __float_as_uint(raw.y), __float_as_uint(raw.z), __float_as_uint(raw.w)};
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      v[2 * c] += __uint_as_float(u[c] << 16);
      v[2 * c + 1] += __uint_as_float(u[c] & 0xffff0000u);
    }
  }
  // `bias8`: the lane's 8 bias values, the same for every row it emits.  Loaded once with the prefetch: a
  // load inside this function would wait on the memory counter, which also counts the stores of the
  // previous call, and so serialise the eight store rounds of a wave.
  __device__ __forceinline__ void emit_fast(const DmaP &p, int m, int nn, float (&v)[8], const Pre &r,
                                            const float4 &bias8) const {
    if (p.bias) add_bf16x8(v, bias8);
    if (p.res && p.res_fp32) {
      v[0] += r.lo.x; v[1] += r.lo.y; v[2] += r.lo.z; v[3] += r.lo.w;
      v[4] += r.hi.x; v[5] += r.hi.y; v[6] += r.hi.z; v[7] += r.hi.w;
    } else if (p.res) {
      add_bf16x8(v, r.lo);
    }
    const int64_t ci = int64_t(m) * p.ldc + nn;
    if (p.c_fp32) {
      float *c = static_cast<float *>(p.C) + ci;
      float4 lo = *reinterpret_cast<float4 *>(v), hi = *reinterpret_cast<float4 *>(v + 4);
      if (p.accumulate) {
        if (p.res) {   // the prefetch slot held the residual: read C now
          const float4 a = *reinterpret_cast<const float4 *>(c), b = *reinterpret_cast<const float4 *>(c + 4);
          lo.x += a.x; lo.y += a.y; lo.z += a.z; lo.w += a.w;
          hi.x += b.x; hi.y += b.y; hi.z += b.z; hi.w += b.w;
        } else {
          lo.x += r.lo.x; lo.y += r.lo.y; lo.z += r.lo.z; lo.w += r.lo.w;
          hi.x += r.hi.x; hi.y += r.hi.y; hi.z += r.hi.z; hi.w += r.hi.w;
        }
      }
      *reinterpret_cast<float4 *>(c) = lo;
      *reinterpret_cast<float4 *>(c + 4) = hi;
    } else {
      Vec16<bf16_t> o;
#pragma unroll
      for (int k = 0; k < 8; ++k) o.v[k] = from_f32<bf16_t>(v[k]);
      // gelu_out == C: only the activation is wanted (a forward pass that keeps nothing for a backward pass)
      if (p.gelu_out != static_cast<bf16_t *>(p.C)) store16(static_cast<bf16_t *>(p.C) + ci, o);
      if (p.gelu_out) {
        Vec16<bf16_t> g;
#pragma unroll
        for (int k = 0; k < 8; ++k) g.v[k] = from_f32<bf16_t>(gelu_fast(to_f32(o.v[k])));
        store16(p.gelu_out + ci, g);
      }
    }
  }
  // one element; src points at its fp32 value in LDS
  __device__ __forceinline__ void emit_one(const DmaP &p, int m, int nn, float v) const {
    if (p.bias) v += to_f32(p.bias[nn]);
    if (p.res)
      v += p.res_fp32 ? reinterpret_cast<const float *>(p.res)[int64_t(m) * p.ldr + nn]
                      : to_f32(p.res[int64_t(m) * p.ldr + nn]);
    const int64_t ci = int64_t(m) * p.ldc + nn;
    if (p.c_fp32) {
      float *c = static_cast<float *>(p.C) + ci;
      *c = p.accumulate ? *c + v : v;
    } else {
      const bf16_t o = from_f32<bf16_t>(v);
      static_cast<bf16_t *>(p.C)[ci] = o;
      if (p.gelu_out) p.gelu_out[ci] = from_f32<bf16_t>(gelu_f(to_f32(o)));
    }
  }
  // a row's group of 8 columns, whose fp32 values lie at src in LDS: in one piece where the group lies inside C,
  // else whatever of it does, element by element
  __device__ __forceinline__ void emit8(const DmaP &p, int m, int nn, const float *src, const Pre &r,
                                        const float4 &bias8) const {
    if (whole8(p, m, nn)) {
      float v[8];
      *reinterpret_cast<float4 *>(v) = *reinterpret_cast<const float4 *>(src);
      *reinterpret_cast<float4 *>(v + 4) = *reinterpret_cast<const float4 *>(src + 4);
      emit_fast(p, m, nn, v, r, bias8);
    } else if (m < p.M) {
#pragma unroll 1
      for (int k = 0; k < 8; ++k)
        if (nn + k < p.N) emit_one(p, m, nn + k, src[k]);
    }
  }
};

template <bool TA, bool TB, int BK, int S>
__global__ __launch_bounds__(NT) void k_gemm_dma(DmaP p, int tiles_per_split, int grid_n, int splits) {
  extern __shared__ __attribute__((aligned(1024))) bf16_t smem[];
  constexpr int TILE = BM * BK;            // elements per operand per stage
  constexpr int L = 2 * (BK / 16);         // load-to-LDS instructions per thread per K tile
  static_assert(S >= 3, "the tile being fetched gets its last part after the barrier: two tiles must be ahead of it");
  static_assert((S - 1) * L <= 63, "vmcnt is a 6-bit counter");
  const int tid = threadIdx.x, lane = tid % 64;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
  const int wm = wave / 2, wn = wave % 2;
  // Workgroup b runs on XCD b % 8, each with an L2 of its own.  Without a split of the contraction: XCD x gets
  // the x-th contiguous range of tile ids (ranges differ by at most one), tiles ordered in bands of 8 tile rows
  // walked column by column, so that neighbours in time share operand tiles in that L2.  With a split (few
  // tiles, long K): the split index varies fastest, so an XCD works on ONE K range of every tile and each
  // byte of A and B is fetched by one XCD only (with the tile fastest, every XCD streamed all of A).
  int bid = blockIdx.x, split_idx = 0;
  const int nb = gridDim.x / splits, grid_m = nb / grid_n;
  if (splits > 1) {
    split_idx = bid % splits;
    bid /= splits;
  } else {
    const int x = bid % 8, per = nb / 8, extra = nb % 8;
    bid = x * per + min(x, extra) + bid / 8;
  }
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

  const int nk_all = p.K / BK;
  const int kt0 = split_idx * tiles_per_split;
  const int n = min(nk_all, kt0 + tiles_per_split) - kt0;   // K tiles of this workgroup
  Dma<TA, BK> da;
  Dma<TB, BK> db;
  da.init(p.lda, m0, p.M, lane, wave);
  db.init(p.ldb, n0, p.N, lane, wave);
  const uint32_t lds0 = uint32_t(reinterpret_cast<uintptr_t>(smem));
  // element strides of one K tile in each operand
  const uint64_t a_kstep = TA ? uint64_t(BK) * p.lda : uint64_t(BK);
  const uint64_t b_kstep = TB ? uint64_t(BK) * p.ldb : uint64_t(BK);
  const bf16_t *a_next = p.A + uint64_t(kt0) * a_kstep;
  const bf16_t *b_next = p.B + uint64_t(kt0) * b_kstep;
  auto issue = [&](int stage) {
    da.issue(a_next, lds0 + uint32_t(stage) * uint32_t(4 * TILE), wave);
    db.issue(b_next, lds0 + uint32_t(stage) * uint32_t(4 * TILE) + uint32_t(2 * TILE), wave);
    a_next += a_kstep;
    b_next += b_kstep;
  };
#pragma unroll
  for (int s = 0; s < S; ++s)
    if (s < n) issue(s);

  const int arow = wm * 64, brow = wn * 64;
  constexpr int KS = BK / 16;
  // operand fragments: read one step ahead of their multiplies (two buffers) with K tiles
  // of 32, two steps ahead (four buffers, indexed by the step within the tile) with 64
  constexpr int NBUF = KS == 4 ? 4 : 2;
  bf16x8 fa[NBUF][2], fb[NBUF][2];
  auto load_frags = [&](int buf, int stage, int ks) {
    const bf16_t *a_s = smem + stage * (2 * TILE), *b_s = a_s + TILE;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      fa[buf][i] = frag<TA, BK>(a_s, arow + 32 * i, ks, lane);
      fb[buf][i] = frag<TB, BK>(b_s, brow + 32 * i, ks, lane);
    }
  };
  // tile 0 has landed once at most the S-1 tiles issued after it are outstanding
  if (n > S - 1) wait_vm<(S - 1) * L>();
  else wait_vm<0>();
  __syncthreads();
  if (n > 0) {
    load_frags(0, 0, 0);
    if (KS == 4) load_frags(1, 0, 1);
  }
  // One 16-deep step: the four multiplies on fragment buffer `cur`, each followed by one
  // of the four fragment reads of a later step (into buffer `nxt`) and, twice, by one
  // load-to-LDS of the tile being fetched.  A wavefront issues in order and an LDS read
  // occupies its issue slot for some 20 cycles, so reads grouped in front of the
  // multiplies would delay them; placed behind a multiply each read issues while the
  // matrix pipe works through that multiply's 32 cycles.  The fences pin this order.
#define HMY_FENCE() __builtin_amdgcn_sched_barrier(0)
  auto step = [&](int cur, int nxt, bool reads, int nstage, int nks, bool fetch, int fstage, int part) {
    const bf16_t *a_s = smem + nstage * (2 * TILE), *b_s = a_s + TILE;
    const uint32_t fl = lds0 + uint32_t(fstage) * uint32_t(4 * TILE);
    HMY_FENCE();
    acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][0], fb[cur][0], acc[0][0], 0, 0, 0);
    HMY_FENCE();
    if (reads) fa[nxt][0] = frag<TA, BK>(a_s, arow, nks, lane);
    HMY_FENCE();
    acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][0], fb[cur][1], acc[0][1], 0, 0, 0);
    HMY_FENCE();
    if (reads) fb[nxt][0] = frag<TB, BK>(b_s, brow, nks, lane);
    if (fetch) da.issue_one(a_next, fl, wave, part);
    HMY_FENCE();
    acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][1], fb[cur][0], acc[1][0], 0, 0, 0);
    HMY_FENCE();
    if (reads) fb[nxt][1] = frag<TB, BK>(b_s, brow + 32, nks, lane);
    HMY_FENCE();
    acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][1], fb[cur][1], acc[1][1], 0, 0, 0);
    HMY_FENCE();
    if (reads) fa[nxt][1] = frag<TA, BK>(a_s, arow + 32, nks, lane);
    if (fetch) db.issue_one(b_next, fl + uint32_t(2 * TILE), wave, part);
    HMY_FENCE();
  };
  int stage = 0;      // stage holding tile t
  int freed = S - 1;  // stage of tile t-1: free since the barrier inside that tile
  const bool split = splits > 1;
  Epi e;
  e.init(p, m0, n0);
  const int m_tile = m0 + wm * 64, n_tile = n0 + wn * 64;
  Epi::Pre pre[2][4];
  float4 bias8 = make_float4(0.f, 0.f, 0.f, 0.f);
  // lane's share of the output: slab i (32 rows), pass q -> row 8 q + lane/8, columns 8 (lane%8) .. +7
  auto prefetch_outputs = [&]() {
    if (split || !e.fast) return;
    if (p.bias && (e.inside || n_tile + 8 * (lane % 8) + 8 <= p.N))
      bias8 = *reinterpret_cast<const float4 *>(p.bias + n_tile + 8 * (lane % 8));
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q) e.prefetch(p, m_tile + 32 * i + 8 * q + lane / 8, n_tile + 8 * (lane % 8), pre[i][q]);
  };
  if constexpr (KS == 4) {
    for (int t = 0; t + 1 < n; ++t) {
      const int next = stage + 1 == S ? 0 : stage + 1;
      // tile t+S-1 goes to the stage tile t-1 has left, a part per step
      const bool fetch = t > 0 && t + S - 1 < n;
      step(0, 2, true, stage, 2, fetch, freed, 0);
      step(1, 3, true, stage, 3, fetch, freed, 1);
      // every read of tile t has been issued.  Tile t+1 has landed once at most the S-3
      // whole tiles issued after it and two parts of the tile being fetched are outstanding.
      if (t + S - 1 < n) wait_vm<(S - 3) * L + 4>();
      else wait_vm<0>();
      __syncthreads();   // tile t+1 visible to every wave; every wave is done reading tile t
      step(2, 0, true, next, 0, fetch, freed, 2);
      step(3, 1, true, next, 1, fetch, freed, 3);
      if (fetch) {
        a_next += a_kstep;
        b_next += b_kstep;
      }
      freed = stage;
      stage = next;
    }
    prefetch_outputs();
    if (n > 0) {   // last tile: nothing left to fetch or wait for
      step(0, 2, true, stage, 2, false, 0, 0);
      step(1, 3, true, stage, 3, false, 0, 0);
      step(2, 0, false, stage, 0, false, 0, 0);
      step(3, 1, false, stage, 0, false, 0, 0);
    }
  } else {
    for (int t = 0; t + 1 < n; ++t) {
      const int next = stage + 1 == S ? 0 : stage + 1;
      const bool fetch = t > 0 && t + S - 1 < n;
#pragma unroll
      for (int ks = 0; ks + 1 < KS; ++ks) step(ks & 1, (ks + 1) & 1, true, stage, ks + 1, fetch, freed, ks);
      // every read of tile t has been issued.  Tile t+1 has landed once at most the S-2
      // tiles issued after it (the one being fetched lacks its last part) are outstanding.
      if (t + S - 1 < n) wait_vm<(S - 2) * L - 2>();
      else wait_vm<0>();
      __syncthreads();   // tile t+1 visible to every wave; every wave is done reading tile t
      step((KS - 1) & 1, 0, true, next, 0, fetch, freed, KS - 1);
      if (fetch) {
        a_next += a_kstep;
        b_next += b_kstep;
      }
      freed = stage;
      stage = next;
    }
    prefetch_outputs();
    if (n > 0) {   // last tile: nothing left to fetch or wait for
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) step(ks & 1, (ks + 1) & 1, ks + 1 < KS, stage, ks + 1, false, 0, 0);
    }
  }
#undef HMY_FENCE

  // Epilogue.  Accumulator register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4,
  // column l%32 of a 32x32 block: stored from there, a wavefront would write 2-byte
  // elements in 64-byte runs.  Each wave instead passes its 64x64 outputs, 32 rows at a
  // time, through 8 KiB of LDS (the operand stages are free now) and leaves with 8
  // consecutive columns per lane: 16-byte stores, 128 contiguous bytes per row.  Rows
  // that differ in bit 2 are written by the two lane halves at once; flipping bit 5 of
  // the column for them keeps the halves on different banks.
  if (split) {   // fp32 atomics: one column per lane, straight from the accumulator layout
    const int m_base = m0 + wm * 64 + 4 * (lane / 32), n_base = n0 + wn * 64 + lane % 32;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int nn = n_base + j * 32;
      if (nn >= p.N) continue;
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = m_base + i * 32 + 8 * (r / 4) + r % 4;
          if (m < p.M) atomicAdd(static_cast<float *>(p.C) + int64_t(m) * p.ldc + nn, acc[i][j][r]);
        }
    }
    return;
  }
  __syncthreads();   // every wave has finished reading the operand stages
  float *slab = reinterpret_cast<float *>(smem) + wave * 2048;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = 8 * (r / 4) + 4 * (lane / 32) + r % 4, col = 32 * j + lane % 32;
        slab[row * 64 + (col ^ (((row >> 2) & 1) << 5))] = acc[i][j][r];
      }
    if (e.fast) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int row = 8 * q + lane / 8, c0 = 8 * (lane % 8);
        const float *src = slab + row * 64 + (c0 ^ (((row >> 2) & 1) << 5));
        e.emit8(p, m_tile + 32 * i + row, n_tile + c0, src, pre[i][q], bias8);
      }
    } else {
#pragma unroll 1
      for (int idx = lane; idx < 32 * 64; idx += 64) {   // one row of 64 columns per pass
        const int row = idx / 64, col = idx % 64;
        const int m = m_tile + 32 * i + row, nn = n_tile + col;
        if (m < p.M && nn < p.N) e.emit_one(p, m, nn, slab[row * 64 + (col ^ (((row >> 2) & 1) << 5))]);
      }
    }
  }
}

// The same GEMM on a 256x256 block tile for outputs large enough to give every compute unit one: what bounds the
// 128x128 kernel is the rate at which the L2 caches feed the load-to-LDS instructions of all compute units together,
// and a tile of twice the side moves half the bytes per multiply.  Eight waves of 128x64 (4x2 multiplies of 32x32x16
// per 16-deep step, two waves per SIMD) over 128 KiB of LDS: a ring of four stages of K tiles of 32, or two stages of
// K tiles of 64.  With the contraction index contiguous in memory a K tile of 32 takes 64 bytes of every operand
// row, half a cache line, and the other half a tile later, when the line has left the compute unit's cache again;
// a K tile of 64 takes whole lines, and the loads to LDS alone then run a quarter faster.  Two stages mean that a
// tile is requested only when the tile before the one being multiplied has been left by every wave, one tile (64
// multiplies per SIMD) before its first use.  Each operand's 256 rows are kept as two 128-row sub-tiles in the
// layouts of the 128x128 kernel; waves 0-3 copy the first sub-tile of A and of B, waves 4-7 the second, each group
// splitting its sub-tile the way the four waves of that kernel do.
template <bool TA, bool TB, int BK, int S>
__global__ __launch_bounds__(512) void k_gemm_dma256(DmaP p, int grid_n) {
  extern __shared__ __attribute__((aligned(1024))) bf16_t smem[];
  constexpr int BT = 256;
  constexpr int SUB = BM * BK;        // elements of one 128-row sub-tile
  constexpr int STAGE = 4 * SUB;      // elements of one stage: A rows 0-127, A rows 128-255, B likewise
  constexpr int NJ = BK / 16;         // load-to-LDS instructions per thread, operand and K tile
  constexpr int L = 2 * NJ;           // load-to-LDS instructions per thread per K tile
  constexpr int KS = BK / 16;         // 16-deep steps per K tile
  static_assert(S >= 2, "one stage is multiplied while the others are in flight");
  static_assert((S - 1) * L <= 63, "vmcnt is a 6-bit counter");
  static_assert(S * STAGE * 2 >= 128 * 1024, "the output stage needs 16 KiB of LDS per wave");
  const int tid = threadIdx.x, lane = tid % 64;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
  const int wm = wave / 4, wn = wave % 4;     // this wave's outputs: rows 128 wm .. +127, columns 64 wn .. +63
  const int half = wave / 4, w4 = wave % 4;   // the sub-tile of each operand this wave copies, and its share of it
  // workgroup -> tile as in the 128x128 kernel (the contraction is never split here: the fp32 atomics of a split
  // make the sum's order, and with it a result that is rounded afterwards, differ from run to run)
  int bid = blockIdx.x;
  const int nb = gridDim.x, grid_m = nb / grid_n;
  {
    const int x = bid % 8, per = nb / 8, extra = nb % 8;
    bid = x * per + min(x, extra) + bid / 8;
  }
  constexpr int kBand = 4;
  const int band = bid / (kBand * grid_n), first_m = band * kBand;
  const int band_rows = min(grid_m - first_m, kBand);
  const int in_band = bid - band * kBand * grid_n;
  const int m0 = (first_m + in_band % band_rows) * BT, n0 = (in_band / band_rows) * BT;

  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int n = p.K / BK;   // K tiles
  Dma<TA, BK> da;
  Dma<TB, BK> db;
  da.init(p.lda, m0 + BM * half, p.M, lane, w4);
  db.init(p.ldb, n0 + BM * half, p.N, lane, w4);
  const uint32_t lds0 = uint32_t(reinterpret_cast<uintptr_t>(smem));
  const uint32_t a_off = uint32_t(half) * uint32_t(2 * SUB), b_off = uint32_t(4 * SUB) + a_off;   // bytes inside a stage
  const uint64_t a_kstep = TA ? uint64_t(BK) * p.lda : uint64_t(BK);
  const uint64_t b_kstep = TB ? uint64_t(BK) * p.ldb : uint64_t(BK);
  const bf16_t *a_next = p.A, *b_next = p.B;
#pragma unroll
  for (int s = 0; s < S; ++s)
    if (s < n) {
      da.issue(a_next, lds0 + uint32_t(s) * uint32_t(2 * STAGE) + a_off, w4);
      db.issue(b_next, lds0 + uint32_t(s) * uint32_t(2 * STAGE) + b_off, w4);
      a_next += a_kstep;
      b_next += b_kstep;
    }

  const int a_sub = wm * SUB, b_sub = 2 * SUB + (wn / 2) * SUB, brow = (wn % 2) * 64;
  bf16x8 fa[2][4], fb[2][2];   // fragments of one 16-deep step, read one step ahead of their multiplies
  if (n > S - 1) wait_vm<(S - 1) * L>();
  else wait_vm<0>();
  __syncthreads();
  if (n > 0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) fa[0][i] = frag<TA, BK>(smem + a_sub, 32 * i, 0, lane);
#pragma unroll
    for (int j = 0; j < 2; ++j) fb[0][j] = frag<TB, BK>(smem + b_sub, brow + 32 * j, 0, lane);
  }
#define HMY_FENCE() __builtin_amdgcn_sched_barrier(0)
#define HMY_MFMA(i, j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][i], fb[cur][j], acc[i][j], 0, 0, 0)
  // One 16-deep step: eight multiplies on fragment buffer `cur`; behind six of them one of the six fragment reads of the
  // next step (from stage `nstage`, step `nks`, into buffer `nxt`); with `fetch`, the load-to-LDS instructions that
  // bring the next tile into stage `fstage`, one behind a multiply each: four of them (K tile 32) behind the last
  // five multiplies, eight (K tile 64) behind all.
  auto step = [&](int cur, int nxt, bool reads, int nstage, int nks, bool fetch, int fstage) {
    const bf16_t *a_s = smem + nstage * STAGE + a_sub, *b_s = smem + nstage * STAGE + b_sub;
    const uint32_t fl = lds0 + uint32_t(fstage) * uint32_t(2 * STAGE);
    // slot k = behind the k-th multiply
    auto fetch_slot = [&](int k) {
      if (!fetch) return;
      const int i = NJ == 2 ? k - 3 : k;   // which of the tile's L instructions
      if (i < 0 || i >= L) return;
      if (i % 2 == 0) da.issue_one(a_next, fl + a_off, w4, i / 2);
      else db.issue_one(b_next, fl + b_off, w4, i / 2);
    };
    HMY_FENCE();
    HMY_MFMA(0, 0);
    HMY_FENCE();
    if (reads) fa[nxt][0] = frag<TA, BK>(a_s, 0, nks, lane);
    fetch_slot(0);
    HMY_FENCE();
    HMY_MFMA(0, 1);
    HMY_FENCE();
    if (reads) fb[nxt][0] = frag<TB, BK>(b_s, brow, nks, lane);
    fetch_slot(1);
    HMY_FENCE();
    HMY_MFMA(1, 0);
    HMY_FENCE();
    if (reads) fb[nxt][1] = frag<TB, BK>(b_s, brow + 32, nks, lane);
    fetch_slot(2);
    HMY_FENCE();
    HMY_MFMA(1, 1);
    HMY_FENCE();
    if (reads) fa[nxt][1] = frag<TA, BK>(a_s, 32, nks, lane);
    fetch_slot(3);
    HMY_FENCE();
    HMY_MFMA(2, 0);
    HMY_FENCE();
    if (reads) fa[nxt][2] = frag<TA, BK>(a_s, 64, nks, lane);
    fetch_slot(4);
    HMY_FENCE();
    HMY_MFMA(2, 1);
    HMY_FENCE();
    if (reads) fa[nxt][3] = frag<TA, BK>(a_s, 96, nks, lane);
    fetch_slot(5);
    HMY_FENCE();
    HMY_MFMA(3, 0);
    HMY_FENCE();
    fetch_slot(6);
    HMY_FENCE();
    HMY_MFMA(3, 1);
    HMY_FENCE();
    fetch_slot(7);
    HMY_FENCE();
  };
  int stage = 0;      // stage holding tile t
  Epi e;
  e.init(p, m0, n0, BT);
  const int m_tile = m0 + wm * 128, n_tile = n0 + wn * 64;
  // what the output stage adds, fetched one 32-row slab ahead: slab i, pass q -> row 32 i + 8 q + lane/8, columns 8 (lane%8) .. +7
  Epi::Pre pre[2][4];
  float4 bias8 = make_float4(0.f, 0.f, 0.f, 0.f);
  auto prefetch_slab = [&](int i, int buf) {
#pragma unroll
    for (int q = 0; q < 4; ++q) e.prefetch(p, m_tile + 32 * i + 8 * q + lane / 8, n_tile + 8 * (lane % 8), pre[buf][q]);
  };
  for (int t = 0; t + 1 < n; ++t) {
    const int next = stage + 1 == S ? 0 : stage + 1;
#pragma unroll
    for (int ks = 0; ks + 1 < KS; ++ks) step(ks % 2, (ks + 1) % 2, true, stage, ks + 1, false, 0);
    // every read of tile t has been issued.  Tiles up to t+S-1 have been requested: tile t+1 has landed once at most
    // the S-2 behind it are outstanding.
    if (t + S - 1 < n) wait_vm<(S - 2) * L>();
    else wait_vm<0>();
    __syncthreads();   // tile t+1 visible to every wave; every wave is done reading tile t
    const bool fetch = t + S < n;   // tile t+S goes to the stage tile t has just left: S-1 tiles ahead of its use
    step((KS - 1) % 2, 0, true, next, 0, fetch, stage);
    if (fetch) {
      a_next += a_kstep;
      b_next += b_kstep;
    }
    stage = next;
  }
  if (e.fast) {
    if (p.bias && (e.inside || n_tile + 8 * (lane % 8) + 8 <= p.N))
      bias8 = *reinterpret_cast<const float4 *>(p.bias + n_tile + 8 * (lane % 8));
    prefetch_slab(0, 0);
  }
  if (n > 0) {   // last tile: nothing left to fetch or wait for
#pragma unroll
    for (int ks = 0; ks + 1 < KS; ++ks) step(ks % 2, (ks + 1) % 2, true, stage, ks + 1, false, 0);
    step((KS - 1) % 2, 0, false, stage, 0, false, 0);
  }
#undef HMY_MFMA
#undef HMY_FENCE

  // output stage as in the 128x128 kernel: 32 rows at a time through LDS, alternating between two 8 KiB buffers per
  // wave so that one slab's stores to memory overlap the next slab's way through LDS
  __syncthreads();   // every wave has finished reading the operand stages
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float *slab = reinterpret_cast<float *>(smem) + wave * 4096 + (i & 1) * 2048;
    if (e.fast && i + 1 < 4) prefetch_slab(i + 1, (i + 1) & 1);
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = 8 * (r / 4) + 4 * (lane / 32) + r % 4, col = 32 * j + lane % 32;
        slab[row * 64 + (col ^ (((row >> 2) & 1) << 5))] = acc[i][j][r];
      }
    if (e.fast) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int row = 8 * q + lane / 8, c0 = 8 * (lane % 8);
        const float *src = slab + row * 64 + (c0 ^ (((row >> 2) & 1) << 5));
        e.emit8(p, m_tile + 32 * i + row, n_tile + c0, src, pre[i & 1][q], bias8);
      }
    } else {
#pragma unroll 1
      for (int idx = lane; idx < 32 * 64; idx += 64) {   // one row of 64 columns per pass
        const int row = idx / 64, col = idx % 64;
        const int m = m_tile + 32 * i + row, nn = n_tile + col;
        if (m < p.M && nn < p.N) e.emit_one(p, m, nn, slab[row * 64 + (col ^ (((row >> 2) & 1) << 5))]);
      }
    }
  }
}

inline int check_launch(const char *what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(HMY_E_HIP, "launch of %s failed: %s", what, hipGetErrorString(e));
  return HMY_OK;
}

template <int BK, int S>
int launch_cfg(const hmy_gemm_desc &g, const DmaP &p, dim3 grid, int tiles_per_split, int gn, int splits, hipStream_t s) {
  const size_t lds = size_t(S) * 2 * BM * BK * sizeof(bf16_t);
  dim3 block(NT);
  if (!g.ta && !g.tb) hipLaunchKernelGGL((k_gemm_dma<false, false, BK, S>), grid, block, lds, s, p, tiles_per_split, gn, splits);
  else if (!g.ta && g.tb) hipLaunchKernelGGL((k_gemm_dma<false, true, BK, S>), grid, block, lds, s, p, tiles_per_split, gn, splits);
  else if (g.ta && !g.tb) hipLaunchKernelGGL((k_gemm_dma<true, false, BK, S>), grid, block, lds, s, p, tiles_per_split, gn, splits);
  else hipLaunchKernelGGL((k_gemm_dma<true, true, BK, S>), grid, block, lds, s, p, tiles_per_split, gn, splits);
  return check_launch("gemm_dma");
}

template <int BK, int S>
int launch_cfg256(const hmy_gemm_desc &g, const DmaP &p, dim3 grid, int gn, hipStream_t s) {
  const size_t lds = size_t(S) * 4 * BM * BK * sizeof(bf16_t);
  dim3 block(512);
  if (!g.ta && !g.tb) hipLaunchKernelGGL((k_gemm_dma256<false, false, BK, S>), grid, block, lds, s, p, gn);
  else if (!g.ta && g.tb) hipLaunchKernelGGL((k_gemm_dma256<false, true, BK, S>), grid, block, lds, s, p, gn);
  else if (g.ta && !g.tb) hipLaunchKernelGGL((k_gemm_dma256<true, false, BK, S>), grid, block, lds, s, p, gn);
  else hipLaunchKernelGGL((k_gemm_dma256<true, true, BK, S>), grid, block, lds, s, p, gn);
  return check_launch("gemm_dma256");
}

int env_int(const char *name, int dflt) {
  const char *v = std::getenv(name);
  return v ? std::atoi(v) : dflt;
}

}  // namespace

// Shapes this kernel takes: K a multiple of 32 (no K tail: the copy engine cannot
// mask), 16-byte aligned operands with leading dimensions that are multiples of 8
// elements, every operand spanning less than 4 GiB (32-bit byte offsets).
bool gemm_dma_eligible(const hmy_gemm_desc &g) {
  const int64_t a_span = int64_t(g.ta ? g.K : g.M) * g.lda, b_span = int64_t(g.tb ? g.K : g.N) * g.ldb;
  return g.K % 32 == 0 && a_span < (int64_t(1) << 31) && b_span < (int64_t(1) << 31);
}

int launch_gemm_dma(const hmy_gemm_desc &g, stream_t st) {
  DmaP p;
  p.A = static_cast<const bf16_t *>(g.A); p.B = static_cast<const bf16_t *>(g.B); p.C = g.C;
  p.bias = static_cast<const bf16_t *>(g.bias); p.res = static_cast<const bf16_t *>(g.res);
  p.gelu_out = static_cast<bf16_t *>(g.gelu_out);
  p.M = g.M; p.N = g.N; p.K = g.K;
  p.lda = uint32_t(g.lda); p.ldb = uint32_t(g.ldb); p.ldc = g.ldc; p.ldr = g.ldr;
  p.c_fp32 = g.c_fp32; p.accumulate = g.accumulate; p.res_fp32 = g.res_fp32;
  static const int force_bk = env_int("HMY_GEMM_BK", 0), force_s = env_int("HMY_GEMM_STAGES", 0);
  static const int force_tile = env_int("HMY_GEMM_TILE", 0);   // 128 | 256: that block tile for every shape it can take
  const bool can_split = g.accumulate && g.c_fp32 && !g.bias && !g.res;
  {
    // 256x256 tiles when they still give most compute units a workgroup (and a second round, if there is one, is
    // at least half full): half the operand bytes per multiply through the L2 caches.  Measured: 152 such tiles
    // (2048 x 4800 x 1600) 49 against 57 us, 175 (1600 x 6400 x 2048) 71 against 72 us, 64 much slower.
    const int gm2 = (g.M + 255) / 256, gn2 = (g.N + 255) / 256, wgs = gm2 * gn2;
    const bool fills = wgs >= 144 && (wgs <= 256 || wgs >= 384);
    if (force_tile != 128 && g.M >= 256 && g.N >= 256 && (force_tile == 256 || fills)) {
      // K tiles of 64 where an operand has the contraction index contiguous (whole cache lines of its rows)
      bool deep = (!g.ta || !g.tb) && g.K % 64 == 0;
      if (force_bk == 32 || (force_bk == 64 && g.K % 64 == 0)) deep = force_bk == 64;
      return deep ? launch_cfg256<64, 2>(g, p, dim3(wgs), gn2, (hipStream_t)st)
                  : launch_cfg256<32, 4>(g, p, dim3(wgs), gn2, (hipStream_t)st);
    }
  }
  const int gm = (g.M + BM - 1) / BM, gn = (g.N + BM - 1) / BM;
  // split the contraction over workgroups (fp32 atomics into C) only while that fills
  // idle compute units: with one workgroup per unit already, a deeper K loop beats more
  // workgroups that each pay a prologue and an atomic epilogue
  int splits = 1;
  if (can_split && gm * gn <= 128)
    splits = std::max(1, std::min(256 / (gm * gn), g.K / 256));
  // few workgroups: one per compute unit, deep K tiles and a deep ring; many: smaller
  // stages so that several are resident and overlap each other's prologue and epilogue
  int bk = g.K % 64 == 0 && gm * gn * splits <= 256 ? 64 : 32;
  if (force_bk == 32 || (force_bk == 64 && g.K % 64 == 0)) bk = force_bk;
  int stages = 4;
  if (force_s >= 3 && force_s <= 4) stages = force_s;
  const int nk = g.K / bk;
  const int tps = (nk + splits - 1) / splits;
  splits = (nk + tps - 1) / tps;
  dim3 grid(gm * gn * splits);
  hipStream_t s = (hipStream_t)st;
  if (bk == 64) {
    if (stages == 3) return launch_cfg<64, 3>(g, p, grid, tps, gn, splits, s);
    return launch_cfg<64, 4>(g, p, grid, tps, gn, splits, s);
  }
  if (stages == 3) return launch_cfg<32, 3>(g, p, grid, tps, gn, splits, s);
  return launch_cfg<32, 4>(g, p, grid, tps, gn, splits, s);
}

}  // namespace hmy
