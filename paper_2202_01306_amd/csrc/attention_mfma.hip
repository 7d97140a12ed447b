// bf16 flash attention on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16).
//
// Every kernel keeps the scores transposed so that one lane owns one softmax row:
// for S^T = K Q^T the 32x32 accumulator gives lane l the query l%32 and sixteen of
// the 32 keys (the lane 32 further holds the other sixteen), so row maxima and sums
// are register reductions plus one cross-lane exchange, and the per-row rescaling
// of the output accumulator (also transposed: O^T = V^T P^T) is a per-lane scalar.
// Operands that must be read along the "wrong" axis of their LDS tile (V^T, K^T,
// dO^T, Q^T) come through ds_read_b64_tr_b16, which hands each lane four values
// from four different tile rows; the contraction order this induces (rows
// 4h+0..3 then 8+4h+0..3 of each group of 16, h = lane/32) is exactly the order in
// which the accumulator of the preceding MFMA holds them, so probabilities go from
// accumulator to operand without leaving registers.
//
// qkv is [T, 3d] with q | k | v thirds, head h at columns h*DH..; lse is [b,H,s].
// HMY_ATTN_SPLIT=0 (read once per process) runs the forward pass at head dimension 64 on the four-wave kernel
// instead of the eight-wave one, for timing the two against each other.
#include <cstdlib>

#include "dev_common.h"
#include "hmy_internal.h"

namespace hmy {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;       // 4 wavefronts, 32 rows of the block tile each
// At least two waves per SIMD, i.e. at most 256 registers per lane: the compiler then keeps the MFMA
// accumulators in ordinary vector registers.  Left free to use the accumulation registers it moved the
// score and output tiles back and forth with v_accvgpr_read / write around every softmax and rescaling
// (about 100 extra vector instructions per 32 x 32 subtile in kernels that are bound by exactly those).
// The dK/dV kernel at head dimension 128 needs more than 256 registers and keeps the default.
#define HMY_MFMA_IN_VGPRS __attribute__((amdgpu_waves_per_eu(2)))
constexpr int kBlockRows = 128;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <int DH> struct Cfg {
  static constexpr int TILE = DH == 128 ? 32 : 64;   // rows of the streamed tiles
  static constexpr int PITCH = DH + 8;               // padded LDS row (conflict-free 16-byte reads)
  static constexpr int KSTEPS = DH / 16;             // MFMA k-steps along the head dimension
  static constexpr int DTILES = DH / 32;             // 32-row output tiles along the head dimension
};

__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int r = 0; r < 16; ++r) z[r] = 0.f;
  return z;
}
__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Stage ROWS rows x DH columns (global row stride ld) into LDS [ROWS][PITCH]; rows at
// or beyond n_valid are zero.  Two phases, so that the loads of the next tile are in
// flight while the current one is multiplied: fetch into registers, put into LDS after
// the compute.
template <int DH, int ROWS, int NT = kThreads>
struct TileRegs {
  static constexpr int CPR = DH / 8;
  static constexpr int N = ROWS * CPR / NT;
  static_assert(N >= 1 && ROWS * CPR % NT == 0, "tile does not divide over the workgroup");
  Vec16<bf16_t> v[N];
  __device__ __forceinline__ void fetch(const bf16_t *src, int64_t ld, int n_valid, int tid) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int q = tid + i * NT, r = q / CPR, c = (q % CPR) * 8;
      if (r < n_valid) {
        v[i] = load16(src + int64_t(r) * ld + c);
      } else {
#pragma unroll
        for (int k = 0; k < 8; ++k) v[i].v[k] = bf16_t(0.f);
      }
    }
  }
  __device__ __forceinline__ void put(bf16_t *lds, int tid) const {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int q = tid + i * NT, r = q / CPR, c = (q % CPR) * 8;
      store16(lds + r * Cfg<DH>::PITCH + c, v[i]);
    }
  }
};

// Operand fragment along a tile row: lane (row%32, kg) gets 8 consecutive columns.
template <int DH>
__device__ __forceinline__ bf16x8 frag_row(const bf16_t *lds, int row, int col) {
  return *reinterpret_cast<const bf16x8 *>(lds + row * Cfg<DH>::PITCH + col);
}
// Operand fragment across tile rows (the tile transposed): the lane's MFMA row is tile
// column colbase + lane%32; its 8 contraction slots are tile rows rowbase + 4h + 0..3
// and rowbase + 8 + 4h + 0..3 (h = lane/32).
template <int DH>
__device__ __forceinline__ bf16x8 frag_col(const bf16_t *lds, int rowbase, int colbase, int lane) {
  const int s = lane % 16, g16 = (lane / 16) % 2, h = lane / 32;
  const bf16_t *p = lds + (rowbase + 4 * h + s / 4) * Cfg<DH>::PITCH + colbase + 16 * g16 + 4 * (s % 4);
  typedef __attribute__((address_space(3))) short4v *lds_ptr;
  const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
  const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 8 * Cfg<DH>::PITCH));
  union { short4v s4[2]; bf16x8 b; } u;
  u.s4[0] = lo;
  u.s4[1] = hi;
  return u.b;
}
// Fragment straight from global memory: row-major matrix, lane (row, kg) gets columns col..col+7.
__device__ __forceinline__ bf16x8 frag_global(const bf16_t *base, int64_t ld, int row, int col) {
  return *reinterpret_cast<const bf16x8 *>(base + int64_t(row) * ld + col);
}
// Accumulator registers 8c..8c+7 as an operand fragment (rows 16c+4h+0..3, 16c+8+4h+0..3).
__device__ __forceinline__ bf16x8 acc_to_frag(const f32x16 &a, int c) {
  bf16x8 f;
#pragma unroll
  for (int k = 0; k < 8; ++k) f[k] = static_cast<__bf16>(a[8 * c + k]);
  return f;
}
// tile row (0..31) held in accumulator register r by a lane of half h
__device__ __forceinline__ int acc_row(int r, int h) { return 8 * (r / 4) + 4 * h + r % 4; }

// db[c] += sum over the workgroup's 128 rows of the values stored from the accumulators (scaled and rounded to bf16
// as they are stored; rows that are not stored count as zero): the bias gradient of the QKV projection, taken while
// the gradient of its output is still in registers.  acc[t][r] of lane l in wave w belongs to row 32 w + l % 32,
// column 32 t + 8 (r / 4) + 4 (l / 32) + r % 4.  The values pass through LDS, 64 columns at a time (rows padded to
// an odd number of floats so that the lanes of a wave, which hold different rows, fall on different banks); every
// thread then adds up a share of one column, and one atomic per thread leaves the workgroup -- a few wide atomic
// instructions instead of one narrow one per value and wave.  Every thread of the workgroup must call this.
constexpr int kBiasCols = 64, kBiasPitch = kBiasCols + 1;
template <int NT>
__device__ __forceinline__ void bias_grad_sums(float *db, const f32x16 (&acc)[NT], float scale, bool row_stored, float *lds,
                                               int tid) {
  const int lane = tid % 64, h = lane / 32, row = 32 * (tid / 64) + lane % 32;
  constexpr int G = NT < 2 ? NT : 2, W = 32 * G;   // accumulator tiles and columns per pass
#pragma unroll
  for (int g = 0; g < NT; g += G) {
#pragma unroll
    for (int t = 0; t < G; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        lds[row * kBiasPitch + 32 * t + 8 * (r / 4) + 4 * h + r % 4] =
            row_stored ? static_cast<float>(static_cast<__bf16>(acc[g + t][r] * scale)) : 0.f;
    __syncthreads();
    const int col = tid % W, part = tid / W;
    constexpr int kParts = kThreads / W;
    float sum = 0.f;
    for (int rr = part; rr < kBlockRows; rr += kParts) sum += lds[rr * kBiasPitch + col];
    atomicAdd(db + 32 * g + col, sum);
    __syncthreads();
  }
}

// Which 128-row block, head and sequence a workgroup takes (1-D grid of nrb * H * b workgroups).
// With a causal mask the work of a row block grows with the number of keys (queries) it sees, from 1
// to nrb units.  Workgroups are handed out in linear order, round-robin over the 8 XCDs, and a launch
// of the usual size is resident all at once (about two workgroups per compute unit), so the order IS
// the placement: a grid with the row block in its fastest dimension puts every heaviest block on one
// XCD and pairs equal weights on a compute unit (16 units on some, 2 on others, where 9 would do).
// Here the (row block, head, sequence) triples are ranked by weight, heaviest first, and dealt out in
// rounds of one workgroup per compute unit, every other round backwards: a unit that got a heavy block
// in one round gets a light one in the next, and each XCD sees every weight equally often.
struct BlockCoord { int rb, head, seq; };
__device__ __forceinline__ BlockCoord block_coord(int nrb, int H, int causal, bool heaviest_is_last_row_block) {
  const int n = gridDim.x, l = blockIdx.x, bh_count = n / nrb;
  int r = l;
  if (causal) {
    constexpr int kUnits = 256;
    const int round = l / kUnits, first = round * kUnits, len = min(kUnits, n - first);
    if (round & 1) r = first + (len - 1 - (l - first));
  }
  const int rank = r / bh_count, bh = r % bh_count;
  BlockCoord c;
  c.rb = !causal ? rank : (heaviest_is_last_row_block ? nrb - 1 - rank : rank);
  c.head = bh % H;
  c.seq = bh / H;
  return c;
}

// ---------------------------------------------------------------------------------
// Forward.  grid (ceil(s/128) * H * b).  Wave w owns queries q0 + 32w .. +31.
template <int DH>
__global__ __launch_bounds__(kThreads) HMY_MFMA_IN_VGPRS void k_attn_fwd_mfma(const bf16_t *qkv, bf16_t *o, float *lse, int s, int H,
                                                            int causal) {
  typedef Cfg<DH> C;
  __shared__ __attribute__((aligned(16))) bf16_t sK[2][C::TILE * C::PITCH];
  __shared__ __attribute__((aligned(16))) bf16_t sV[2][C::TILE * C::PITCH];
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64, h2 = lane / 32;
  const int d = H * DH;
  const int64_t ld = 3 * int64_t(d);
  const BlockCoord bc = block_coord((s + kBlockRows - 1) / kBlockRows, H, causal, true);   // the last query blocks see the most keys
  const int head = bc.head, seq = bc.seq, q0 = bc.rb * kBlockRows;
  const bf16_t *base = qkv + int64_t(seq) * s * ld + head * DH;
  const int qw = q0 + 32 * wave;                 // first query of this wave
  const int q = qw + lane % 32;                  // this lane's query
  const int q_ld = min(q, s - 1);
  bf16x8 fq[C::KSTEPS];
#pragma unroll
  for (int c = 0; c < C::KSTEPS; ++c) fq[c] = frag_global(base, ld, q_ld, 16 * c + 8 * h2);
  f32x16 acc_o[C::DTILES];
#pragma unroll
  for (int t = 0; t < C::DTILES; ++t) acc_o[t] = zero16();
  // Row sums come out of the matrix cores as well: a row of ones in the role of V^T makes every
  // register of acc_l the sum over keys of this lane's query's probabilities (both half-waves' keys),
  // which takes sixteen additions per 32 keys off the vector ALU, the unit this kernel is bound by.
  f32x16 acc_l = zero16();
  bf16x8 ones;
#pragma unroll
  for (int k = 0; k < 8; ++k) ones[k] = static_cast<__bf16>(1.f);
  // m_run is the REFERENCE the exponentials are taken against, not the exact running maximum: it is
  // raised (and everything accumulated rescaled) only when some row's scores outgrow it by more than
  // kSlack, so probabilities stay below 2^kSlack and most tiles skip the rescaling altogether
  constexpr float kSlack = 8.f;
  float m_run = -INFINITY;
  const float sc = rsqrtf(float(DH)) * kLog2e;   // scores in log2 units
  const int k_end = causal ? min(s, q0 + kBlockRows) : s;
  const int n_tiles = (k_end + C::TILE - 1) / C::TILE;
  TileRegs<DH, C::TILE> rk, rv;
  rk.fetch(base + d, ld, min(C::TILE, s), tid);
  rv.fetch(base + 2 * d, ld, min(C::TILE, s), tid);
  rk.put(sK[0], tid);
  rv.put(sV[0], tid);
  __syncthreads();
  for (int kt = 0; kt < n_tiles; ++kt) {
    const int cur = kt & 1, k0 = kt * C::TILE;
    const bool more = kt + 1 < n_tiles;
    if (more) {   // next tile's loads fly during this tile's multiplies
      const int kn = k0 + C::TILE;
      rk.fetch(base + d + int64_t(kn) * ld, ld, min(C::TILE, s - kn), tid);
      rv.fetch(base + 2 * d + int64_t(kn) * ld, ld, min(C::TILE, s - kn), tid);
    }
    const bool wave_active = !causal || k0 <= qw + 31;   // some query of this wave sees this tile
    if (wave_active) {
      // The 32-key subtiles of the tile go through each stage together: their score products are independent chains
      // of multiplies that overlap, the row maximum and the decision to rescale are taken once over all of them, and
      // the exponentials of one overlap the multiplies of another.  A subtile that lies wholly past this wave's
      // queries (second half of a diagonal tile) is carried along fully masked: its probabilities are exact zeros.
      constexpr int NS = C::TILE / 32;
      f32x16 st[NS];
#pragma unroll
      for (int sub = 0; sub < NS; ++sub) st[sub] = zero16();
      // S^T[key, query] = K Q^T
#pragma unroll
      for (int c = 0; c < C::KSTEPS; ++c)
#pragma unroll
        for (int sub = 0; sub < NS; ++sub)
          st[sub] = mfma(frag_row<DH>(sK[cur], 32 * sub + lane % 32, 16 * c + 8 * h2), fq[c], st[sub]);
#pragma unroll
      for (int sub = 0; sub < NS; ++sub) {
        const int kb = k0 + 32 * sub;                     // first key of the 32-key subtile
        // keys past the sequence end or (causal) past the query: only the diagonal and
        // the last subtile need the per-element test
        if (kb + 32 > s || (causal && kb + 31 > qw)) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = kb + acc_row(r, h2);
            if (!(key < s && (!causal || key <= q))) st[sub][r] = -INFINITY;
          }
        }
      }
      float mx = st[0][0];
#pragma unroll
      for (int sub = 0; sub < NS; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, st[sub][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * sc;     // log2 units (sc > 0)
      if (__any(mx > m_run + kSlack)) {   // some row outgrew its reference: raise it, rescale what was accumulated
        const float m_new = fmaxf(m_run, mx);
        const float corr = m_new == -INFINITY ? 1.f : fast_exp2(m_run - m_new);
        acc_l[0] *= corr;
#pragma unroll
        for (int t = 0; t < C::DTILES; ++t)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc_o[t][r] *= corr;
        m_run = m_new;
      }
      // rows that have seen no key yet keep m = -inf; use 0 as the reference to stay finite
      const float m_ref = m_run == -INFINITY ? 0.f : m_run;
#pragma unroll
      for (int sub = 0; sub < NS; ++sub) {
#pragma unroll
        for (int r = 0; r < 16; ++r) st[sub][r] = fast_exp2(fmaf(st[sub][r], sc, -m_ref));
        // O^T[dh, query] += V^T P^T, and the row sums
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          const bf16x8 fp = acc_to_frag(st[sub], c);
#pragma unroll
          for (int t = 0; t < C::DTILES; ++t)
            acc_o[t] = mfma(frag_col<DH>(sV[cur], 32 * sub + 16 * c, 32 * t, lane), fp, acc_o[t]);
          acc_l = mfma(ones, fp, acc_l);
        }
      }
    }
    if (more) {
      rk.put(sK[cur ^ 1], tid);
      rv.put(sV[cur ^ 1], tid);
    }
    __syncthreads();
  }
  const float l_tot = acc_l[0];
  if (q < s) {
    const float inv = 1.f / l_tot;
    bf16_t *orow = o + (int64_t(seq) * s + q) * d + head * DH;
#pragma unroll
    for (int t = 0; t < C::DTILES; ++t)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        bf16x4 v;
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = static_cast<__bf16>(acc_o[t][4 * j + k] * inv);
        *reinterpret_cast<bf16x4 *>(orow + 32 * t + 8 * j + 4 * h2) = v;
      }
    if (h2 == 0) lse[(int64_t(seq) * H + head) * s + q] = (m_run + log2f(l_tot)) * kLn2;
  }
}

// ---------------------------------------------------------------------------------
// Forward for key tiles of two 32-key subtiles (head dimensions up to 64): eight waves per workgroup.  Wave w takes
// the queries q0 + 32 (w % 4) .. + 31 and, of every key tile, only subtile w / 4: two waves share each group of
// queries and split its keys, each with a running reference, row sum and output accumulator of its own, which the
// pair merges through LDS at the end.  The same work in twice as many, half as long chains: the kernel is bound by
// each wave's serial chain (multiplies, maximum, exponentials, multiplies), and with four waves per SIMD instead of
// two the vector unit of one wave works while the matrix unit of another does.
template <int DH>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(4))) void k_attn_fwd_mfma_split(const bf16_t *qkv, bf16_t *o, float *lse, int s, int H,
                                                                                                    int causal) {
  typedef Cfg<DH> C;
  static_assert(C::TILE == 64, "two subtiles per key tile");
  constexpr int NTHR = 512;
  constexpr int kTileElems = C::TILE * C::PITCH;
  // K and V tiles, double buffered; afterwards the same bytes carry one wave's state to its partner
  __shared__ __attribute__((aligned(16))) bf16_t smem[4 * kTileElems];
  static_assert(4 * kTileElems * 2 >= 4 * 64 * (2 + 16 * C::DTILES) * 4, "the merge needs 2 + 16 DTILES floats per lane of four waves");
  auto sK = [&](int buf) { return smem + buf * kTileElems; };
  auto sV = [&](int buf) { return smem + (2 + buf) * kTileElems; };
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64, h2 = lane / 32;
  const int rg = wave % 4, sub = wave / 4;
  const int d = H * DH;
  const int64_t ld = 3 * int64_t(d);
  const BlockCoord bc = block_coord((s + kBlockRows - 1) / kBlockRows, H, causal, true);
  const int head = bc.head, seq = bc.seq, q0 = bc.rb * kBlockRows;
  const bf16_t *base = qkv + int64_t(seq) * s * ld + head * DH;
  const int qw = q0 + 32 * rg, q = qw + lane % 32, q_ld = min(q, s - 1);
  bf16x8 fq[C::KSTEPS];
#pragma unroll
  for (int c = 0; c < C::KSTEPS; ++c) fq[c] = frag_global(base, ld, q_ld, 16 * c + 8 * h2);
  f32x16 acc_o[C::DTILES];
#pragma unroll
  for (int t = 0; t < C::DTILES; ++t) acc_o[t] = zero16();
  f32x16 acc_l = zero16();   // row sums from the matrix cores, as in the kernel above
  bf16x8 ones;
#pragma unroll
  for (int k = 0; k < 8; ++k) ones[k] = static_cast<__bf16>(1.f);
  constexpr float kSlack = 8.f;   // the exponent reference is raised only when a row outgrows it by this much
  float m_run = -INFINITY;
  const float sc = rsqrtf(float(DH)) * kLog2e;   // scores in log2 units
  const int k_end = causal ? min(s, q0 + kBlockRows) : s;
  const int n_tiles = (k_end + C::TILE - 1) / C::TILE;
  TileRegs<DH, C::TILE, NTHR> rk, rv;
  rk.fetch(base + d, ld, min(C::TILE, s), tid);
  rv.fetch(base + 2 * d, ld, min(C::TILE, s), tid);
  rk.put(sK(0), tid);
  rv.put(sV(0), tid);
  __syncthreads();
  for (int kt = 0; kt < n_tiles; ++kt) {
    const int cur = kt & 1, k0 = kt * C::TILE;
    const bool more = kt + 1 < n_tiles;
    if (more) {   // next tile's loads fly during this tile's multiplies
      const int kn = k0 + C::TILE;
      rk.fetch(base + d + int64_t(kn) * ld, ld, min(C::TILE, s - kn), tid);
      rv.fetch(base + 2 * d + int64_t(kn) * ld, ld, min(C::TILE, s - kn), tid);
    }
    const int kb = k0 + 32 * sub;   // first key of this wave's subtile
    if (kb < s && (!causal || kb <= qw + 31)) {   // some query of this wave sees some key of it
      // S^T[key, query] = K Q^T
      f32x16 st = zero16();
#pragma unroll
      for (int c = 0; c < C::KSTEPS; ++c)
        st = mfma(frag_row<DH>(sK(cur), 32 * sub + lane % 32, 16 * c + 8 * h2), fq[c], st);
      if (kb + 32 > s || (causal && kb + 31 > qw)) {   // ragged or diagonal subtile: per-element test
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kb + acc_row(r, h2);
          if (!(key < s && (!causal || key <= q))) st[r] = -INFINITY;
        }
      }
      float mx = st[0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, st[r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * sc;     // log2 units (sc > 0)
      if (__any(mx > m_run + kSlack)) {   // some row outgrew its reference: raise it, rescale what was accumulated
        const float m_new = fmaxf(m_run, mx);
        const float corr = m_new == -INFINITY ? 1.f : fast_exp2(m_run - m_new);
        acc_l[0] *= corr;
#pragma unroll
        for (int t = 0; t < C::DTILES; ++t)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc_o[t][r] *= corr;
        m_run = m_new;
      }
      const float m_ref = m_run == -INFINITY ? 0.f : m_run;   // a row that has seen no key yet
#pragma unroll
      for (int r = 0; r < 16; ++r) st[r] = fast_exp2(fmaf(st[r], sc, -m_ref));
      // O^T[dh, query] += V^T P^T, and the row sums
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const bf16x8 fp = acc_to_frag(st, c);
#pragma unroll
        for (int t = 0; t < C::DTILES; ++t)
          acc_o[t] = mfma(frag_col<DH>(sV(cur), 32 * sub + 16 * c, 32 * t, lane), fp, acc_o[t]);
        acc_l = mfma(ones, fp, acc_l);
      }
    }
    if (more) {
      rk.put(sK(cur ^ 1), tid);
      rv.put(sV(cur ^ 1), tid);
    }
    __syncthreads();
  }
  // merge the two key subsets of each query: the wave of the second subtile hands over its reference, row sum and
  // accumulator ([value][lane] floats: conflict-free both ways); the first rescales both to the larger reference
  constexpr int NV = 2 + 16 * C::DTILES;
  float *xch = reinterpret_cast<float *>(smem) + rg * (NV * 64);
  if (sub == 1) {
    xch[lane] = m_run;
    xch[64 + lane] = acc_l[0];
#pragma unroll
    for (int t = 0; t < C::DTILES; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) xch[(2 + 16 * t + r) * 64 + lane] = acc_o[t][r];
  }
  __syncthreads();
  if (sub == 1) return;
  const float m_b = xch[lane], l_b = xch[64 + lane];
  const float m_tot = fmaxf(m_run, m_b);   // finite: the first subtile of the first tile holds key 0, which every query sees
  const float ca = fast_exp2(m_run - m_tot), cb = m_b == -INFINITY ? 0.f : fast_exp2(m_b - m_tot);
  const float l_tot = acc_l[0] * ca + l_b * cb;
  if (q < s) {
    const float inv = 1.f / l_tot;
    bf16_t *orow = o + (int64_t(seq) * s + q) * d + head * DH;
#pragma unroll
    for (int t = 0; t < C::DTILES; ++t)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        bf16x4 v;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int r = 4 * j + k;
          v[k] = static_cast<__bf16>((acc_o[t][r] * ca + xch[(2 + 16 * t + r) * 64 + lane] * cb) * inv);
        }
        *reinterpret_cast<bf16x4 *>(orow + 32 * t + 8 * j + 4 * h2) = v;
      }
    if (h2 == 0) lse[(int64_t(seq) * H + head) * s + q] = (m_tot + log2f(l_tot)) * kLn2;
  }
}

// ---------------------------------------------------------------------------------
// dQ.  grid (ceil(s/128), H, b).  Wave w owns queries q0+32w..; K and V tiles stream.
// Also delta[seq,head,q] = sum_c dO[q,c] * O[q,c], which this kernel needs per query and the dK/dV kernel, launched
// behind it, reads per streamed query row: each lane holds half of its query's dO row as multiply operands already, so
// the sum is 4 DH / 16 multiply-adds and one exchange with the lane that holds the other half, and no kernel of its own.
template <int DH>
__global__ __launch_bounds__(kThreads) HMY_MFMA_IN_VGPRS void k_attn_bwd_dq_mfma(const bf16_t *qkv, const bf16_t *o, const bf16_t *d_o,
                                                               const float *lse, float *delta, bf16_t *dqkv, float *dbias,
                                                               int s, int H, int causal) {
  typedef Cfg<DH> C;
  __shared__ __attribute__((aligned(16))) bf16_t sK[2][C::TILE * C::PITCH];
  __shared__ __attribute__((aligned(16))) bf16_t sV[2][C::TILE * C::PITCH];
  __shared__ float sB[kBlockRows * kBiasPitch];   // the bias gradient's way through LDS
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64, h2 = lane / 32;
  const int d = H * DH;
  const int64_t ld = 3 * int64_t(d);
  const BlockCoord bc = block_coord((s + kBlockRows - 1) / kBlockRows, H, causal, true);
  const int head = bc.head, seq = bc.seq, q0 = bc.rb * kBlockRows;
  const bf16_t *base = qkv + int64_t(seq) * s * ld + head * DH;
  const bf16_t *gbase = d_o + int64_t(seq) * s * d + head * DH;
  const bf16_t *obase = o + int64_t(seq) * s * d + head * DH;
  const int qw = q0 + 32 * wave, q = qw + lane % 32, q_ld = min(q, s - 1);
  bf16x8 fq[C::KSTEPS], fg[C::KSTEPS];
  float dl = 0.f;
#pragma unroll
  for (int c = 0; c < C::KSTEPS; ++c) {
    fq[c] = frag_global(base, ld, q_ld, 16 * c + 8 * h2);
    fg[c] = frag_global(gbase, d, q_ld, 16 * c + 8 * h2);
    const bf16x8 fo = frag_global(obase, d, q_ld, 16 * c + 8 * h2);
#pragma unroll
    for (int k = 0; k < 8; ++k) dl = fmaf(static_cast<float>(fg[c][k]), static_cast<float>(fo[k]), dl);
  }
  dl += __shfl_xor(dl, 32, 64);   // the other half of the row
  if (h2 == 0 && q < s) delta[(int64_t(seq) * H + head) * s + q] = dl;
  const float L = lse[(int64_t(seq) * H + head) * s + q_ld] * kLog2e;   // log2 units
  const float scale = rsqrtf(float(DH)), sc = scale * kLog2e;
  f32x16 acc_q[C::DTILES];
#pragma unroll
  for (int t = 0; t < C::DTILES; ++t) acc_q[t] = zero16();
  const int k_end = causal ? min(s, q0 + kBlockRows) : s;
  const int n_tiles = (k_end + C::TILE - 1) / C::TILE;
  TileRegs<DH, C::TILE> rk, rv;
  rk.fetch(base + d, ld, min(C::TILE, s), tid);
  rv.fetch(base + 2 * d, ld, min(C::TILE, s), tid);
  rk.put(sK[0], tid);
  rv.put(sV[0], tid);
  __syncthreads();
  for (int kt = 0; kt < n_tiles; ++kt) {
    const int cur = kt & 1, k0 = kt * C::TILE;
    const bool more = kt + 1 < n_tiles;
    if (more) {   // next tile's loads fly during this tile's multiplies
      const int kn = k0 + C::TILE;
      rk.fetch(base + d + int64_t(kn) * ld, ld, min(C::TILE, s - kn), tid);
      rv.fetch(base + 2 * d + int64_t(kn) * ld, ld, min(C::TILE, s - kn), tid);
    }
    if (!causal || k0 <= qw + 31) {
#pragma unroll
      for (int sub = 0; sub < C::TILE / 32; ++sub) {
        const int kb = k0 + 32 * sub;
        if (causal && kb > qw + 31) continue;
        f32x16 st = zero16(), dp = zero16();
#pragma unroll
        for (int c = 0; c < C::KSTEPS; ++c) {
          st = mfma(frag_row<DH>(sK[cur], 32 * sub + lane % 32, 16 * c + 8 * h2), fq[c], st);   // S^T = K Q^T
          dp = mfma(frag_row<DH>(sV[cur], 32 * sub + lane % 32, 16 * c + 8 * h2), fg[c], dp);   // dP^T = V dO^T
        }
        if (kb + 32 > s || (causal && kb + 31 > qw)) {   // diagonal or ragged subtile: per-element test
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = kb + acc_row(r, h2);
            const bool ok = key < s && (!causal || key <= q);
            const float p = ok ? fast_exp2(fmaf(st[r], sc, -L)) : 0.f;
            st[r] = p * (dp[r] - dl);                                                             // dS^T
          }
        } else {
#pragma unroll
          for (int r = 0; r < 16; ++r) st[r] = fast_exp2(fmaf(st[r], sc, -L)) * (dp[r] - dl);
        }
        // dQ^T[dh, query] += K^T dS^T
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          const bf16x8 fs = acc_to_frag(st, c);
#pragma unroll
          for (int t = 0; t < C::DTILES; ++t)
            acc_q[t] = mfma(frag_col<DH>(sK[cur], 32 * sub + 16 * c, 32 * t, lane), fs, acc_q[t]);
        }
      }
    }
    if (more) {
      rk.put(sK[cur ^ 1], tid);
      rv.put(sV[cur ^ 1], tid);
    }
    __syncthreads();
  }
  if (q < s) {
    bf16_t *row = dqkv + (int64_t(seq) * s + q) * ld + head * DH;
#pragma unroll
    for (int t = 0; t < C::DTILES; ++t)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        bf16x4 v;
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = static_cast<__bf16>(acc_q[t][4 * j + k] * scale);
        *reinterpret_cast<bf16x4 *>(row + 32 * t + 8 * j + 4 * h2) = v;
      }
  }
  if (dbias) bias_grad_sums<C::DTILES>(dbias + head * DH, acc_q, scale, q < s, sB, tid);
}

// ---------------------------------------------------------------------------------
// dK, dV.  grid (ceil(s/128), H, b).  Wave w owns keys j0+32w..; Q and dO tiles stream.
template <int DH>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(DH == 128 ? 1 : 2))) void k_attn_bwd_dkv_mfma(const bf16_t *qkv, const bf16_t *d_o, const float *lse,
                                                                const float *delta, bf16_t *dqkv, float *dbias, int s,
                                                                int H, int causal) {
  typedef Cfg<DH> C;
  __shared__ __attribute__((aligned(16))) bf16_t sQ[2][C::TILE * C::PITCH];
  __shared__ __attribute__((aligned(16))) bf16_t sG[2][C::TILE * C::PITCH];
  __shared__ __attribute__((aligned(16))) float sL[2][C::TILE], sD[2][C::TILE];
  __shared__ float sB[kBlockRows * kBiasPitch];   // the bias gradient's way through LDS
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64, h2 = lane / 32;
  const int d = H * DH;
  const int64_t ld = 3 * int64_t(d);
  const BlockCoord bc = block_coord((s + kBlockRows - 1) / kBlockRows, H, causal, false);   // the first key blocks are seen by the most queries
  const int head = bc.head, seq = bc.seq, j0 = bc.rb * kBlockRows;
  const bf16_t *base = qkv + int64_t(seq) * s * ld + head * DH;
  const bf16_t *gbase = d_o + int64_t(seq) * s * d + head * DH;
  const float *lbase = lse + (int64_t(seq) * H + head) * s, *dbase = delta + (int64_t(seq) * H + head) * s;
  const int jw = j0 + 32 * wave, key = jw + lane % 32, key_ld = min(key, s - 1);
  bf16x8 fk[C::KSTEPS], fv[C::KSTEPS];
#pragma unroll
  for (int c = 0; c < C::KSTEPS; ++c) {
    fk[c] = frag_global(base + d, ld, key_ld, 16 * c + 8 * h2);
    fv[c] = frag_global(base + 2 * d, ld, key_ld, 16 * c + 8 * h2);
  }
  const float scale = rsqrtf(float(DH)), sc = scale * kLog2e;
  f32x16 acc_k[C::DTILES], acc_v[C::DTILES];
#pragma unroll
  for (int t = 0; t < C::DTILES; ++t) { acc_k[t] = zero16(); acc_v[t] = zero16(); }
  // causal: queries before the block's first key see none of its keys
  const int t_begin = causal ? j0 / C::TILE : 0;
  const int n_tiles = (s + C::TILE - 1) / C::TILE;
  TileRegs<DH, C::TILE> rq, rg;
  float rl = 0.f, rd = 0.f;
  auto fetch = [&](int i0) {
    const int nv = min(C::TILE, s - i0);
    rq.fetch(base + int64_t(i0) * ld, ld, nv, tid);
    rg.fetch(gbase + int64_t(i0) * d, d, nv, tid);
    if (tid < C::TILE) {
      rl = tid < nv ? lbase[i0 + tid] * kLog2e : 0.f;
      rd = tid < nv ? dbase[i0 + tid] : 0.f;
    }
  };
  auto put = [&](int buf) {
    rq.put(sQ[buf], tid);
    rg.put(sG[buf], tid);
    if (tid < C::TILE) {
      sL[buf][tid] = rl;
      sD[buf][tid] = rd;
    }
  };
  if (t_begin < n_tiles) {
    fetch(t_begin * C::TILE);
    put(0);
  }
  __syncthreads();
  for (int it = t_begin; it < n_tiles; ++it) {
    const int cur = (it - t_begin) & 1, i0 = it * C::TILE;
    const bool more = it + 1 < n_tiles;
    // (no register prefetch across the compute here: with both accumulator sets it would
    // cost the second resident wave per SIMD)
    if (more) {
      fetch(i0 + C::TILE);
      put(cur ^ 1);
    }
#pragma unroll
    for (int sub = 0; sub < C::TILE / 32; ++sub) {
      const int ib = i0 + 32 * sub;                       // first query of the subtile
      if (causal && ib + 31 < jw) continue;               // every query precedes every key of this wave
      // S[query, key] = Q K^T and dP[query, key] = dO V^T: lane owns a key, registers run over queries
      f32x16 sm = zero16(), dp = zero16();
#pragma unroll
      for (int c = 0; c < C::KSTEPS; ++c) {
        sm = mfma(frag_row<DH>(sQ[cur], 32 * sub + lane % 32, 16 * c + 8 * h2), fk[c], sm);
        dp = mfma(frag_row<DH>(sG[cur], 32 * sub + lane % 32, 16 * c + 8 * h2), fv[c], dp);
      }
      // queries past the sequence end or (causal) before the key: only the diagonal and
      // the last subtile need the per-element test
      const bool edge = ib + 32 > s || (causal && ib < jw + 31);
      // the lane's sixteen queries are four runs of four consecutive rows: 16-byte reads
      float ql[16], qd[16];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        *reinterpret_cast<float4 *>(ql + 4 * g) = *reinterpret_cast<const float4 *>(&sL[cur][32 * sub + 8 * g + 4 * h2]);
        *reinterpret_cast<float4 *>(qd + 4 * g) = *reinterpret_cast<const float4 *>(&sD[cur][32 * sub + 8 * g + 4 * h2]);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int qi = 32 * sub + acc_row(r, h2);         // query inside the tile
        const bool ok = !edge || (i0 + qi < s && (!causal || key <= i0 + qi));
        const float p = ok ? fast_exp2(fmaf(sm[r], sc, -ql[r])) : 0.f;
        sm[r] = p;                                        // P
        dp[r] = p * (dp[r] - qd[r]);                      // dS
      }
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const bf16x8 fp = acc_to_frag(sm, c), fs = acc_to_frag(dp, c);
#pragma unroll
        for (int t = 0; t < C::DTILES; ++t) {
          acc_v[t] = mfma(frag_col<DH>(sG[cur], 32 * sub + 16 * c, 32 * t, lane), fp, acc_v[t]);   // dV^T += dO^T P
          acc_k[t] = mfma(frag_col<DH>(sQ[cur], 32 * sub + 16 * c, 32 * t, lane), fs, acc_k[t]);   // dK^T += Q^T dS
        }
      }
    }
    __syncthreads();
  }
  if (key < s) {
    bf16_t *row = dqkv + (int64_t(seq) * s + key) * ld + head * DH;
#pragma unroll
    for (int t = 0; t < C::DTILES; ++t)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        bf16x4 vk, vv;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          vk[k] = static_cast<__bf16>(acc_k[t][4 * j + k] * scale);
          vv[k] = static_cast<__bf16>(acc_v[t][4 * j + k]);
        }
        *reinterpret_cast<bf16x4 *>(row + d + 32 * t + 8 * j + 4 * h2) = vk;
        *reinterpret_cast<bf16x4 *>(row + 2 * d + 32 * t + 8 * j + 4 * h2) = vv;
      }
  }
  if (dbias) {
    bias_grad_sums<C::DTILES>(dbias + d + head * DH, acc_k, scale, key < s, sB, tid);
    bias_grad_sums<C::DTILES>(dbias + 2 * d + head * DH, acc_v, 1.f, key < s, sB, tid);
  }
}

inline int check_launch(const char *what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(HMY_E_HIP, "launch of %s failed: %s", what, hipGetErrorString(e));
  return HMY_OK;
}

template <int DH>
int fwd_t(const void *qkv, void *o, float *lse, int b, int s, int H, int causal, hipStream_t st) {
  const dim3 grid(((s + kBlockRows - 1) / kBlockRows) * H * b);
  static const bool split = std::getenv("HMY_ATTN_SPLIT") == nullptr || std::atoi(std::getenv("HMY_ATTN_SPLIT")) != 0;
  if constexpr (DH == 64) {   // two 32-key subtiles per key tile, and enough 16-byte pieces in a tile for 512 threads
    if (split) {
      hipLaunchKernelGGL((k_attn_fwd_mfma_split<DH>), grid, dim3(512), 0, st, (const bf16_t *)qkv, (bf16_t *)o, lse, s, H,
                         causal);
      return check_launch("attn_fwd_mfma_split");
    }
  }
  hipLaunchKernelGGL((k_attn_fwd_mfma<DH>), grid, dim3(kThreads), 0, st, (const bf16_t *)qkv, (bf16_t *)o, lse, s, H,
                     causal);
  return check_launch("attn_fwd_mfma");
}
template <int DH>
int bwd_t(const void *qkv, const void *o, const void *d_o, const float *lse, float *delta, void *dqkv, float *dbias, int b,
          int s, int H, int causal, hipStream_t st) {
  const dim3 grid(((s + kBlockRows - 1) / kBlockRows) * H * b);
  hipLaunchKernelGGL((k_attn_bwd_dq_mfma<DH>), grid, dim3(kThreads), 0, st, (const bf16_t *)qkv, (const bf16_t *)o,
                     (const bf16_t *)d_o, lse, delta, (bf16_t *)dqkv, dbias, s, H, causal);   // writes delta for the next kernel
  hipLaunchKernelGGL((k_attn_bwd_dkv_mfma<DH>), grid, dim3(kThreads), 0, st, (const bf16_t *)qkv, (const bf16_t *)d_o,
                     lse, delta, (bf16_t *)dqkv, dbias, s, H, causal);
  return check_launch("attn_bwd_mfma");
}

}  // namespace

int launch_attn_fwd_mfma(const void *qkv, void *o, float *lse, int b, int s, int H, int dh, int causal, stream_t st) {
  if (dh == 32) return fwd_t<32>(qkv, o, lse, b, s, H, causal, (hipStream_t)st);
  if (dh == 64) return fwd_t<64>(qkv, o, lse, b, s, H, causal, (hipStream_t)st);
  if (dh == 128) return fwd_t<128>(qkv, o, lse, b, s, H, causal, (hipStream_t)st);
  return fail(HMY_E_INVALID, "attention: unsupported head dim %d", dh);
}
int launch_attn_bwd_mfma(const void *qkv, const void *o, const void *d_o, const float *lse, float *delta, void *dqkv,
                         float *dbias, int b, int s, int H, int dh, int causal, stream_t st) {
  if (dh == 32) return bwd_t<32>(qkv, o, d_o, lse, delta, dqkv, dbias, b, s, H, causal, (hipStream_t)st);
  if (dh == 64) return bwd_t<64>(qkv, o, d_o, lse, delta, dqkv, dbias, b, s, H, causal, (hipStream_t)st);
  if (dh == 128) return bwd_t<128>(qkv, o, d_o, lse, delta, dqkv, dbias, b, s, H, causal, (hipStream_t)st);
  return fail(HMY_E_INVALID, "attention: unsupported head dim %d", dh);
}

}  // namespace hmy
