// Pack planner: per-layer profile, HBM arena layout, balanced-time packing (the paper's
// Algorithm 2, Section 4.3.1) under the HBM budget, the runtime estimate and the
// configuration search of Algorithm 1.
//
// Memory model.  The runtime keeps S weight slots (Section 4.4, prefetch and double
// buffering; S = 3 by default: the pack being computed, the next one arriving, and the
// previous one still draining through its update and write-back), one activation workspace
// for the backward pack in flight, and a pack-independent reserve (resident boundary
// activations, checkpoint rings, gradient scratch, the optimizer ring).  A layer's footprint
// for the packing is therefore
//   forward : S * E * p                   (E bytes per weight, p parameters)
//   backward: S * (E + 4) * p + act       (weights + fp32 gradients per slot; activations once)
// and the capacity is the budget minus the reserve.  Times are nanoseconds per microbatch:
// measured ones if the budget brings them, else flop counts over a sustained rate (integers,
// so the balanced split of equal layers has exact ties).
#include <algorithm>
#include <cstring>
#include <string>

#include "hmy_internal.h"

namespace hmy {

BlockActs block_acts(const hmy_model_spec &s, int micro_batch) {
  const uint64_t E = s.precision == HMY_PREC_BF16 ? 2 : 4;
  const uint64_t T = uint64_t(micro_batch) * s.seq_len, d = s.d_model, f = s.d_ffn, H = s.n_heads;
  BlockActs b;
  uint64_t off = 0;
  auto take = [&](uint64_t bytes) { uint64_t o = off; off += a256(bytes); return o; };
  b.x_in = take(T * d * 4);    // the residual stream is fp32 whatever E is
  b.a = take(T * d * E);
  b.qkv = take(3 * T * d * E);
  b.o = take(T * d * E);
  b.x_mid = take(T * d * 4);
  b.h = take(T * d * E);
  b.u = take(T * f * E);
  b.g = take(T * f * E);
  b.ln1_mean = take(T * 4);
  b.ln1_rstd = take(T * 4);
  b.ln2_mean = take(T * 4);
  b.ln2_rstd = take(T * 4);
  b.lse = take(T * H * 4);
  b.size = off;
  return b;
}

HeadActs head_acts(const hmy_model_spec &s, int micro_batch) {
  const uint64_t E = s.precision == HMY_PREC_BF16 ? 2 : 4;
  const uint64_t T = uint64_t(micro_batch) * s.seq_len, d = s.d_model;
  HeadActs h;
  h.chunk_rows = int(std::min<uint64_t>(T, kLogitRows));
  h.ldl = (int64_t(s.vocab) + 63) / 64 * 64;   // rows start on 128-byte lines (element type) for the GEMMs that read them
  uint64_t off = 0;
  auto take = [&](uint64_t bytes) { uint64_t o = off; off += a256(bytes); return o; };
  h.x_in = take(T * d * 4);
  h.z = take(T * d * E);
  h.mean = take(T * 4);
  h.rstd = take(T * 4);
  h.logits = take(uint64_t(h.chunk_rows) * h.ldl * 4);
  // the gradient of the logits is kept for the whole microbatch: the two GEMMs that consume it then run once
  // per microbatch with T rows instead of once per chunk (the weight-gradient one would otherwise read and write
  // the fp32 [vocab, d] accumulator once per chunk, which is what bounded it)
  h.dlogits = take(T * h.ldl * E);
  h.dz32 = take(T * d * 4);   // fp32 accumulator of the input gradient (its contraction may be split)
  h.size = off;
  return h;
}

int resolve(Packs *p, int n_micro, int micro_batch, Split *out) {
  if (n_micro < 1 || micro_batch < 1) return fail(HMY_E_INVALID, "n_micro and micro_batch must be >= 1");
  if (p->slots == 0) p->slots = kDefaultSlots;
  if (p->distance == 0) p->distance = 1;
  if (p->uF == 0) p->uF = micro_batch;
  if (p->uB == 0) p->uB = micro_batch;
  if (p->slots < 2 || p->slots > kMaxSlots)
    return fail(HMY_E_BAD_SCHEDULE, "weight_slots %d (2..%d)", p->slots, kMaxSlots);
  if (p->distance < 1 || p->distance >= p->slots)
    return fail(HMY_E_BAD_SCHEDULE, "prefetch_distance %d must be at least 1 and below weight_slots %d", p->distance,
                p->slots);
  const int64_t D = int64_t(n_micro) * micro_batch;
  if (D > (1 << 30)) return fail(HMY_E_INVALID, "minibatch too large");
  if (p->uF < 1 || p->uB < 1 || D % p->uF || D % p->uB)
    return fail(HMY_E_BAD_SCHEDULE, "microbatch sizes %d (forward) and %d (backward) must divide the minibatch of %lld "
                "sequences", p->uF, p->uB, (long long)D);
  if (p->order == HMY_ORDER_MICROBATCH_MAJOR && p->uF != p->uB)
    return fail(HMY_E_BAD_SCHEDULE, "the microbatch-major order runs one microbatch list through both passes");
  if (out) *out = Split{int(D), p->uF, p->uB};
  return HMY_OK;
}

Reserved reserved_layout(const Model &m, const Split &sp) {
  const hmy_model_spec &s = m.spec;
  const uint64_t E = m.elem_bytes();
  const uint64_t d = s.d_model, f = s.d_ffn, H = s.n_heads;
  const uint64_t TF = uint64_t(sp.uF) * s.seq_len, TB = uint64_t(sp.uB) * s.seq_len, Tall = uint64_t(sp.D) * s.seq_len;
  Reserved r;
  uint64_t off = 0;
  auto take = [&](uint64_t bytes) { uint64_t o = off; off += a256(bytes); return o; };
  r.x_bytes_F = TF * d * 4;   // the residual stream (boundary activations, their gradients) is fp32
  r.x_bytes_B = TB * d * 4;
  r.ck_bytes_F = TF * d * E;  // checkpoints cross the link rounded to the element type
  r.ck_bytes_B = TB * d * E;
  r.in_bytes = a256(r.ck_bytes_B);
  r.out_bytes = a256(r.ck_bytes_F);
  r.X = take(Tall * d * 4);   // one row per token of the minibatch: either pass's microbatch m is a run of its rows
  r.inring = take(kInRing * r.in_bytes);
  r.outring = take(kOutRing * r.out_bytes);
  r.gbig = take(TB * std::max<uint64_t>(f, 3 * d) * E);
  r.gsmall = take(TB * d * E);
  r.dlow = take(TB * d * E);
  r.delta = take(TB * H * 4);
  r.ids = take(Tall * 4);
  r.targets = take(Tall * 4);
  r.misc = take(4096);
  uint64_t maxp = 0;
  for (int l = 0; l < m.R; ++l) maxp = std::max(maxp, m.params_in(l, l + 1));
  r.k_chunk_params = std::min<uint64_t>(kKChunkMax, maxp);
  r.karr_bytes = a256(r.k_chunk_params * 4);
  r.kring = take(uint64_t(kKRing) * m.k_arrays() * r.karr_bytes);
  r.size = off;
  return r;
}

Rates rates_of(const hmy_budget *b) {
  Rates r;
  if (!b) return r;
  if (b->host_link_MBps) r.link_MBps = b->host_link_MBps;
  if (b->compute_GFLOPs) r.compute_GFLOPs = b->compute_GFLOPs;
  if (b->measured && b->n_measured) {
    r.measured = b->measured;
    r.n_measured = b->n_measured;
  }
  return r;
}

static const hmy_measured_profile *measured_for(const Rates &r, int micro_batch) {
  for (uint32_t i = 0; i < r.n_measured; ++i)
    if (r.measured[i].micro_batch == micro_batch) return &r.measured[i];
  return nullptr;
}

// forward flops of layer l for one microbatch of u sequences
static int64_t layer_flops(const Model &m, int l, int u) {
  const hmy_model_spec &s = m.spec;
  const int64_t T = int64_t(u) * s.seq_len, d = s.d_model, f = s.d_ffn, V = s.vocab;
  if (l == 0) return T * d;
  if (l <= s.n_blocks) return T * (8 * d * d + 4 * d * f + (s.causal ? 2 : 4) * int64_t(s.seq_len) * d);
  return 2 * T * d * V;
}

void layer_profile(const Model &m, const Rates &r, const Split &sp, int slots, std::vector<hmy_layer_profile> *out) {
  const hmy_model_spec &s = m.spec;
  const uint64_t E = m.elem_bytes();
  out->assign(m.R, hmy_layer_profile{});
  const uint64_t act_block = block_acts(s, sp.uB).size;
  const uint64_t act_head = head_acts(s, sp.uB).size;
  const hmy_measured_profile *mF = measured_for(r, sp.uF), *mB = measured_for(r, sp.uB);
  auto ns_of = [&](int64_t flops) { return int64_t((uint64_t(flops) + r.compute_GFLOPs - 1) / r.compute_GFLOPs); };
  for (int l = 0; l < m.R; ++l) {
    hmy_layer_profile &p = (*out)[l];
    p.params = m.params_in(l, l + 1);
    p.flops_fwd = layer_flops(m, l, sp.uF);
    p.ns_fwd = ns_of(p.flops_fwd);
    p.ns_bwd = ns_of(3 * layer_flops(m, l, sp.uB));   // recompute + backward (twice the forward flops)
    // beside link traffic: the measured figure if there is one (never below the time alone), else the same
    auto beside = [](uint64_t alone, uint64_t b) { return int64_t(std::max(alone, b)); };
    int64_t fb = 0, bb = 0;
    if (l == 0) {
      p.act_bwd = 0;
      if (mF) p.ns_fwd = int64_t(mF->embed_fwd_ns), fb = beside(mF->embed_fwd_ns, mF->embed_fwd_beside_ns);
      if (mB)
        p.ns_bwd = int64_t(mB->embed_fwd_ns + mB->embed_bwd_ns),
        bb = beside(mB->embed_fwd_ns, mB->embed_fwd_beside_ns) + beside(mB->embed_bwd_ns, mB->embed_bwd_beside_ns);
    } else if (l <= s.n_blocks) {
      p.act_bwd = act_block;
      if (mF) p.ns_fwd = int64_t(mF->block_fwd_ns), fb = beside(mF->block_fwd_ns, mF->block_fwd_beside_ns);
      if (mB) p.ns_bwd = int64_t(mB->block_bwd_ns), bb = beside(mB->block_bwd_ns, mB->block_bwd_beside_ns);
    } else {
      p.act_bwd = act_head;
      if (mF) p.ns_fwd = int64_t(mF->head_ns), fb = beside(mF->head_ns, mF->head_beside_ns);
      if (mB) p.ns_bwd = int64_t(mB->head_ns), bb = beside(mB->head_ns, mB->head_beside_ns);
    }
    p.ns_fwd_beside = mF ? fb : p.ns_fwd;
    p.ns_bwd_beside = mB ? bb : p.ns_bwd;
    p.mem_fwd = uint64_t(slots) * E * p.params;
    p.mem_bwd = uint64_t(slots) * (E + 4) * p.params + p.act_bwd;
  }
}

uint64_t pack_state_fwd(const Model &m, Pack p) { return a256(m.elem_bytes() * m.params_in(p.a, p.e)); }
uint64_t pack_state_bwd(const Model &m, Pack p) {
  return a256(m.elem_bytes() * m.params_in(p.a, p.e)) + a256(4 * m.params_in(p.a, p.e));
}

Arena arena_layout(const Model &m, const Packs &p, const Split &sp) {
  Arena a;
  a.res = reserved_layout(m, sp);
  a.slots = p.slots;
  const uint64_t act_block = block_acts(m.spec, sp.uB).size, act_head = head_acts(m.spec, sp.uB).size;
  a.slot_bytes = 0;
  a.act_bytes = 0;
  for (const Pack &q : p.fwd) {
    a.slot_bytes = std::max(a.slot_bytes, pack_state_fwd(m, q));
    // a forward task keeps nothing: its blocks share one block's worth of buffers, at the forward microbatch size
    if (q.e > 1) a.act_bytes = std::max(a.act_bytes, block_acts(m.spec, sp.uF).size);
  }
  for (const Pack &q : p.bwd) {
    a.slot_bytes = std::max(a.slot_bytes, pack_state_bwd(m, q));
    uint64_t act = 0;
    for (int l = q.a; l < q.e; ++l) act += l == 0 ? 0 : l <= m.spec.n_blocks ? act_block : act_head;
    a.act_bytes = std::max(a.act_bytes, act);
  }
  for (int i = 0; i < kMaxSlots; ++i) a.slot_off[i] = a.res.size + uint64_t(std::min(i, a.slots - 1)) * a.slot_bytes;
  a.act_off = a.res.size + uint64_t(a.slots) * a.slot_bytes;
  a.total = a.act_off + a.act_bytes;
  return a;
}

std::vector<Region> arena_regions(const Model &m, const Arena &a, const Split &sp) {
  const Reserved &r = a.res;
  const hmy_model_spec &s = m.spec;
  const uint64_t E = m.elem_bytes(), d = s.d_model, Tall = uint64_t(sp.D) * s.seq_len, TB = uint64_t(sp.uB) * s.seq_len;
  std::vector<Region> v;
  v.push_back({"X", r.X, Tall * d * 4});
  v.push_back({"inring", r.inring, kInRing * r.in_bytes});
  v.push_back({"outring", r.outring, kOutRing * r.out_bytes});
  v.push_back({"gbig", r.gbig, TB * std::max<uint64_t>(s.d_ffn, 3 * d) * E});
  v.push_back({"gsmall", r.gsmall, TB * d * E});
  v.push_back({"dlow", r.dlow, TB * d * E});
  v.push_back({"delta", r.delta, TB * uint64_t(s.n_heads) * 4});
  v.push_back({"ids", r.ids, Tall * 4});
  v.push_back({"targets", r.targets, Tall * 4});
  v.push_back({"misc", r.misc, 4096});
  v.push_back({"kring", r.kring, uint64_t(kKRing) * m.k_arrays() * r.karr_bytes});
  for (int i = 0; i < a.slots; ++i) v.push_back({"slot" + std::to_string(i), a.slot_off[i], a.slot_bytes});
  v.push_back({"acts", a.act_off, a.act_bytes});
  return v;
}

int schedule_to_packs(const Model &m, const hmy_schedule *s, Packs *out) {
  if (!s) return fail(HMY_E_INVALID, "null schedule");
  if (s->n_bwd_packs < 1 || s->n_bwd_packs > m.R || s->n_fwd_packs < 0 || s->n_fwd_packs > m.R)
    return fail(HMY_E_BAD_SCHEDULE, "pack counts out of range");
  if (s->order != HMY_ORDER_LAYER_PACK_MAJOR && s->order != HMY_ORDER_MICROBATCH_MAJOR)
    return fail(HMY_E_BAD_SCHEDULE, "unknown task order %d", s->order);
  if (s->update_site != HMY_UPDATE_ON_DEVICE && s->update_site != HMY_UPDATE_ON_HOST)
    return fail(HMY_E_BAD_SCHEDULE, "unknown update site %d", s->update_site);
  if (s->gradients != HMY_GRADIENTS_EXPORTED && s->gradients != HMY_GRADIENTS_ON_DEVICE)
    return fail(HMY_E_BAD_SCHEDULE, "unknown gradient disposal %d", s->gradients);
  if (s->resident_state != HMY_STATE_SWAPPED && s->resident_state != HMY_STATE_RESIDENT_IN_SPARE_BUDGET)
    return fail(HMY_E_BAD_SCHEDULE, "unknown state residency %d", s->resident_state);
  if (s->swap_out != HMY_SWAP_OUT_KERNEL && s->swap_out != HMY_SWAP_OUT_MEMCPY)
    return fail(HMY_E_BAD_SCHEDULE, "unknown swap-out mechanism %d", s->swap_out);
  if (s->weight_slots < 0 || s->prefetch_distance < 0 || s->fwd_micro_batch < 0 || s->bwd_micro_batch < 0)
    return fail(HMY_E_BAD_SCHEDULE, "negative slot count, prefetch distance or microbatch size");
  Packs p;
  p.resident_state = s->resident_state;
  p.order = s->order;
  p.update_site = s->update_site;
  p.gradients = s->gradients;
  p.swap_out = s->swap_out;
  p.slots = s->weight_slots;
  p.distance = s->prefetch_distance;
  p.uF = s->fwd_micro_batch;
  p.uB = s->bwd_micro_batch;
  int pos = 0;
  for (int i = 0; i < s->n_bwd_packs; ++i) {
    int e = s->bwd_pack_end[i];
    if (e <= pos || e > m.R) return fail(HMY_E_BAD_SCHEDULE, "backward pack %d is empty or out of range", i);
    p.bwd.push_back({pos, e});
    pos = e;
  }
  if (pos != m.R) return fail(HMY_E_BAD_SCHEDULE, "backward packs cover %d of %d layers", pos, m.R);
  const int last_start = p.bwd.back().a;
  pos = 0;
  for (int i = 0; i < s->n_fwd_packs; ++i) {
    int e = s->fwd_pack_end[i];
    if (e <= pos || e > last_start) return fail(HMY_E_BAD_SCHEDULE, "forward pack %d is empty or out of range", i);
    p.fwd.push_back({pos, e});
    pos = e;
  }
  if (pos != last_start)
    return fail(HMY_E_BAD_SCHEDULE, "forward packs must cover exactly the %d layers before the last backward pack",
                last_start);
  *out = std::move(p);
  return HMY_OK;
}

void packs_to_schedule(const Packs &p, hmy_schedule *out) {
  std::memset(out, 0, sizeof(*out));
  out->n_fwd_packs = int(p.fwd.size());
  out->n_bwd_packs = int(p.bwd.size());
  out->order = p.order;
  out->update_site = p.update_site;
  out->gradients = p.gradients;
  out->resident_state = p.resident_state;
  out->swap_out = p.swap_out;
  out->weight_slots = p.slots;
  out->prefetch_distance = p.distance;
  out->fwd_micro_batch = p.uF;
  out->bwd_micro_batch = p.uB;
  for (size_t i = 0; i < p.fwd.size(); ++i) out->fwd_pack_end[i] = p.fwd[i].e;
  for (size_t i = 0; i < p.bwd.size(); ++i) out->bwd_pack_end[i] = p.bwd[i].e;
}

// Algorithm 2 on explicit lists over layers first..first+R.  `fits` is the
// whole-packing test ANDed to the per-pack capacity test.  Returns false if not
// even one layer per pack fits.
// The search starts at max(S_min, S_start); *S_used receives the pack count that was
// accepted (R + 1 for the one-layer-per-pack fallback), so that a caller can ask for
// the next feasible candidate.
template <class Fits>
static bool balanced_time_packing(const std::vector<int64_t> &t, const std::vector<uint64_t> &mem,
                                  uint64_t alpha, int first, Fits fits, std::vector<Pack> *out, int S_start = 1,
                                  int *S_used = nullptr) {
  const int R = int(t.size());
  out->clear();
  if (S_used) *S_used = 0;
  if (R == 0) return true;
  if (alpha == 0) return false;
  __int128 total = 0;
  uint64_t msum = 0;
  std::vector<__int128> prefix(R);
  for (int j = 0; j < R; ++j) {
    total += t[j];
    prefix[j] = total;
    msum += mem[j];
  }
  auto per_pack_ok = [&](const std::vector<Pack> &ps) {
    for (const Pack &q : ps) {
      uint64_t s = 0;
      for (int l = q.a; l < q.e; ++l) s += mem[l - first];
      if (s > alpha) return false;
    }
    return true;
  };
  int S_min = int(std::max<uint64_t>(1, (msum + alpha - 1) / alpha));
  for (int S = std::max(S_min, S_start); S <= R; ++S) {
    // cut k = number of layers whose prefix time is <= k * total / S
    std::vector<Pack> ps;
    int prev = 0;
    for (int k = 1; k <= S; ++k) {
      int cut;
      if (k == S) {
        cut = R;
      } else {
        cut = 0;
        for (int j = 0; j < R; ++j)
          if (prefix[j] * S <= __int128(k) * total) ++cut;
      }
      if (cut > prev) ps.push_back({first + prev, first + cut});
      prev = std::max(prev, cut);
    }
    if (per_pack_ok(ps) && fits(ps)) {
      *out = std::move(ps);
      if (S_used) *S_used = S;
      return true;
    }
  }
  if (S_start > R + 1) return false;
  std::vector<Pack> ps;
  for (int j = 0; j < R; ++j) ps.push_back({first + j, first + j + 1});
  if (per_pack_ok(ps) && fits(ps)) {
    *out = std::move(ps);
    if (S_used) *S_used = R + 1;
    return true;
  }
  return false;
}

// Runtime estimate of one iteration for a configuration (the role of the paper's Runtime
// Estimator, Section 4.3.1): an event-driven walk of the task list, in integer nanoseconds,
// over four queues -- the compute stream, the host->device link, the device->host link and,
// with the update on the host, the CPU threads (Section 4.4).  A "visit" is a forward or
// backward task; visit v owns weight slot v mod S.
//   compute  : microbatches of its pass x the sum of its layers' profiled times; needs its weights.
//   weights  : the weights of visit v + distance are requested when visit v starts computing (those
//              of the first `distance` visits at time 0) and need their slot, which the visit S places
//              earlier leaves when its compute ends (forward) or its update has been written back
//              (backward).  The link serves requests in order: one that waits holds up those behind it.
//   stash    : a forward visit's checkpoints go out, a backward visit's come in, while it computes
//              (requested at its start); nothing waits for them, they only occupy the link.
//   update   : when a backward visit's compute ends its optimizer state is requested (host->device)
//              and state, weights and the exported gradient start out (device->host), ending no earlier
//              than the state has arrived; on the host only the gradient goes out and the CPU
//              (about 6 parameters per nanosecond on the machines measured) is one more queue.
//   slowdown : a visit computes for its layers' times alone, stretched towards their times beside link traffic
//              in proportion to the share of it for which the device->host link has work queued at its start.
//   result   : when the last queue falls idle.
uint64_t estimate_iteration_ns(const Model &m, const std::vector<hmy_layer_profile> &prof, const Packs &p,
                               const Split &sp, uint64_t link_MBps) {
  const uint64_t E = m.elem_bytes(), kB = 4 * uint64_t(m.k_arrays());
  auto t_bytes = [&](uint64_t bytes) { return (bytes * 1000 + link_MBps - 1) / link_MBps; };
  const bool host = p.update_site == HMY_UPDATE_ON_HOST;
  const bool export_g = host || p.gradients == HMY_GRADIENTS_EXPORTED;
  constexpr uint64_t kHostParamsPerNs = 6;
  const uint64_t x_all = uint64_t(sp.D) * m.spec.seq_len * m.spec.d_model * E;   // one checkpoint of the whole minibatch
  struct V { bool bwd; uint64_t comp, w, kin, out, cpu, sin, sout, comp_beside; };
  std::vector<V> vs;
  auto is_ckpt = [&](int layer) {
    for (size_t k = 1; k + 1 < p.bwd.size(); ++k)
      if (p.bwd[k].a == layer) return true;
    return false;
  };
  for (const Pack &q : p.fwd) {
    uint64_t ns = 0, nb = 0, n_ck = 0;
    for (int l = q.a; l < q.e; ++l) {
      ns += uint64_t(prof[l].ns_fwd);
      nb += uint64_t(prof[l].ns_fwd_beside);
      n_ck += is_ckpt(l);
    }
    vs.push_back({false, ns * sp.MF(), t_bytes(E * m.params_in(q.a, q.e)), 0, 0, 0, 0, n_ck ? t_bytes(n_ck * x_all) : 0,
                  nb * sp.MF()});
  }
  for (int k = int(p.bwd.size()) - 1; k >= 0; --k) {
    const Pack &q = p.bwd[k];
    uint64_t ns = 0, nb = 0;
    for (int l = q.a; l < q.e; ++l) {
      ns += uint64_t(prof[l].ns_bwd);
      nb += uint64_t(prof[l].ns_bwd_beside);
    }
    const uint64_t P = m.params_in(q.a, q.e);
    const uint64_t sin = (k > 0 && k + 1 < int(p.bwd.size())) ? t_bytes(x_all) : 0;
    if (host) vs.push_back({true, ns * sp.MB(), t_bytes(E * P), 0, t_bytes(4 * P), P / kHostParamsPerNs, sin, 0, nb * sp.MB()});
    else vs.push_back({true, ns * sp.MB(), t_bytes(E * P), t_bytes(kB * P), t_bytes((kB + E + (export_g ? 4 : 0)) * P), 0, sin, 0,
                       nb * sp.MB()});
  }
  const int n = int(vs.size()), S = p.slots, D = p.distance;
  uint64_t h2d_free = 0, d2h_free = 0, comp_free = 0, cpu_free = 0;
  std::vector<uint64_t> w_ready(n, 0), left(n, 0);
  for (int v = 0; v < std::min(D, n); ++v) w_ready[v] = h2d_free = h2d_free + vs[v].w;
  for (int v = 0; v < n; ++v) {
    const uint64_t comp_start = std::max(comp_free, w_ready[v]);
    // the checkpoints a backward visit starts from are its input: it cannot end before they are all in
    uint64_t sin_end = 0;
    if (vs[v].sin) sin_end = h2d_free = std::max(h2d_free, comp_start) + vs[v].sin;
    if (vs[v].sout) d2h_free = std::max(d2h_free, comp_start) + vs[v].sout;
    if (v + D < n) {
      uint64_t s0 = std::max(h2d_free, comp_start);
      if (v + D - S >= 0) s0 = std::max(s0, left[v + D - S]);
      w_ready[v + D] = h2d_free = s0 + vs[v + D].w;
    }
    // kernels run slower while the host-writing update is busy beside them: the visit's time moves from its
    // time alone towards its time beside link traffic, in proportion to the share of it for which the outgoing
    // link still has work queued now (earlier updates, this visit's checkpoints)
    uint64_t comp = vs[v].comp;
    if (vs[v].comp_beside > comp && d2h_free > comp_start) {
      const uint64_t backlog = std::min(d2h_free - comp_start, comp);
      comp += uint64_t((__uint128_t)(vs[v].comp_beside - comp) * backlog / comp);
    }
    const uint64_t comp_end = std::max(comp_start + comp, sin_end);
    comp_free = comp_end;
    if (!vs[v].bwd) {
      left[v] = comp_end;
    } else if (host) {
      const uint64_t out_end = std::max(d2h_free, comp_end) + vs[v].out;
      d2h_free = left[v] = out_end;
      cpu_free = std::max(cpu_free, out_end) + vs[v].cpu;
    } else {
      const uint64_t kin_end = std::max(h2d_free, comp_end) + vs[v].kin;
      h2d_free = kin_end;
      const uint64_t out_end = std::max(std::max(d2h_free, comp_end) + vs[v].out, kin_end);
      d2h_free = left[v] = out_end;
    }
  }
  return std::max(std::max(comp_free, h2d_free), std::max(d2h_free, cpu_free));
}

// The configuration search (Algorithm 1): for every backward microbatch size and slot count the budget
// lets it sweep, backward packs by Algorithm 2, then for every forward microbatch size forward packs by
// Algorithm 2 over the layers before the last backward pack; the configuration with the smallest
// estimated iteration time wins (ties: the earlier one, and candidates are visited with the caller's
// own microbatch size, then the smaller sizes, first).
int plan_packs(const Model &m, const hmy_budget &b, int n_micro, int micro_batch, Packs *out) {
  const uint64_t budget = b.hbm_budget_bytes;
  const Rates rates = rates_of(&b);
  if (b.update_site != HMY_UPDATE_ON_DEVICE && b.update_site != HMY_UPDATE_ON_HOST)
    return fail(HMY_E_INVALID, "budget: unknown update site %u", b.update_site);
  if (n_micro < 1 || micro_batch < 1) return fail(HMY_E_INVALID, "n_micro and micro_batch must be >= 1");
  const int s_lo = b.min_weight_slots ? int(b.min_weight_slots) : kDefaultSlots;
  const int s_hi = b.max_weight_slots ? int(b.max_weight_slots) : std::max(kDefaultSlots, s_lo);
  if (s_lo < 2 || s_hi > kMaxSlots || s_lo > s_hi)
    return fail(HMY_E_INVALID, "budget: weight slots %d..%d (2..%d)", s_lo, s_hi, kMaxSlots);
  const int64_t D = int64_t(n_micro) * micro_batch;
  auto sizes = [&](uint32_t cap) {
    std::vector<int> v = {micro_batch};
    for (int u = 1; u <= int(std::min<int64_t>(cap, D)); ++u)
      if (D % u == 0 && u != micro_batch) v.push_back(u);
    return v;
  };
  const std::vector<int> cand_B = sizes(b.max_bwd_micro_batch), cand_F = sizes(b.max_fwd_micro_batch);
  auto always = [](const std::vector<Pack> &) { return true; };
  bool have = false, reserve_fits = false;
  uint64_t best_ns = 0;
  Packs best;
  auto taper = [](std::vector<Pack> v) {
    const int e = v.front().e;
    if (e < 2) return v;
    std::vector<Pack> head = {{0, 1}, {1, 2}};
    if (e > 2) head.push_back({2, e});
    v.erase(v.begin());
    v.insert(v.begin(), head.begin(), head.end());
    return v;
  };
  for (int uB : cand_B)
    for (int S = s_lo; S <= s_hi; ++S) {
      const Split sB{int(D), uB, uB};
      std::vector<hmy_layer_profile> prof;
      layer_profile(m, rates, sB, S, &prof);
      const Reserved res = reserved_layout(m, sB);
      if (budget <= res.size) continue;
      reserve_fits = true;
      std::vector<int64_t> tb(m.R);
      std::vector<uint64_t> mb(m.R);
      for (int l = 0; l < m.R; ++l) {
        tb[l] = prof[l].ns_bwd;
        mb[l] = prof[l].mem_bwd;
      }
      auto with = [&](const std::vector<Pack> &bwd, int uF) {
        Packs q;
        q.bwd = bwd;
        q.update_site = int(b.update_site);
        q.slots = S;
        q.distance = 1;
        q.uF = uF;
        q.uB = uB;
        return q;
      };
      auto arena_fits = [&](const std::vector<Pack> &bwd) { return arena_layout(m, with(bwd, uB), sB).total <= budget; };
      // One backward packing: for every forward microbatch size, forward packs over the layers before the
      // last backward pack (they share the weight slots sized by the backward packing); each candidate
      // is offered with every prefetch distance its slots allow.
      auto consider = [&](const std::vector<Pack> &bwd) {
        const int RF = bwd.back().a;
        for (int uF : cand_F) {
          const Split sp{int(D), uF, uB};
          Packs p = with(bwd, uF);
          std::vector<hmy_layer_profile> pf;
          layer_profile(m, rates, sp, S, &pf);
          const uint64_t slot = arena_layout(m, p, sp).slot_bytes;
          std::vector<int64_t> tf(RF);
          std::vector<uint64_t> mf(RF);
          for (int l = 0; l < RF; ++l) {
            tf[l] = pf[l].ns_fwd;
            mf[l] = pf[l].mem_fwd;
          }
          if (!balanced_time_packing(tf, mf, uint64_t(S) * slot, 0, always, &p.fwd)) continue;
          auto offer = [&](Packs q) {
            if (arena_layout(m, q, sp).total > budget) return;   // the forward pass's own buffers (another microbatch size)
            for (int dist = 1; dist < S; ++dist) {
              q.distance = dist;
              const uint64_t ns = estimate_iteration_ns(m, pf, q, sp, rates.link_MBps);
              if (!have || ns < best_ns) {
                have = true;
                best_ns = ns;
                best = q;
              }
            }
          };
          offer(p);
          if (b.max_extra_packs > 0 && RF > 2) {
            // the same backward packs with forward packs that double in size from two layers
            // on: the first pack's load is the part of the forward pass nothing can hide
            Packs q = p;
            q.fwd.clear();
            bool ok = true;
            for (int a = 0, size = 2; a < RF; size *= 2) {
              int e = std::min(RF, a + size);
              if (RF - e < size) e = RF;   // a short remainder joins this pack
              uint64_t mem = 0;
              for (int l = a; l < e; ++l) mem += mf[l];
              if (mem > uint64_t(S) * slot) ok = false;
              q.fwd.push_back({a, e});
              a = e;
            }
            if (ok) offer(q);
          }
        }
      };
      // Backward candidates: the first feasible pack count of Algorithm 2 (largest packs), then up to
      // max_extra_packs further feasible pack counts.  When the search is on, each balanced packing is
      // also tried in three reshaped forms that the balanced split cannot produce and the estimate can
      // tell apart:
      //   taper : the first backward pack [0, e) becomes [0,1), [1,2), [2,e) -- the update of
      //           the pack visited last cannot hide behind any compute, so it should be small,
      //           and so should the one before it, which hides behind that short visit;
      //   merge : the last two backward packs become one (if the arena still fits) -- the last
      //           pack is not recomputed, and its layers drop out of the forward pass;
      //   both.
      int S_start = 1;
      for (uint32_t tries = 0; tries <= b.max_extra_packs; ++tries) {
        std::vector<Pack> bwd;
        int S_used = 0;
        if (!balanced_time_packing(tb, mb, budget - res.size, 0, arena_fits, &bwd, S_start, &S_used)) break;
        consider(bwd);
        if (b.max_extra_packs > 0) {
          const std::vector<Pack> t = taper(bwd);
          if (t.size() != bwd.size() && arena_fits(t)) consider(t);
          if (bwd.size() >= 2) {
            std::vector<Pack> g = bwd;
            const Pack last = g.back();
            g.pop_back();
            g.back().e = last.e;
            if (arena_fits(g)) {
              consider(g);
              const std::vector<Pack> tg = taper(g);
              if (tg.size() != g.size() && arena_fits(tg)) consider(tg);
            }
          }
        }
        if (S_used > m.R) break;   // that was the one-layer-per-pack fallback
        S_start = S_used + 1;
      }
    }
  if (!have) {
    if (!reserve_fits)
      return fail(HMY_E_BUDGET_TOO_SMALL, "budget %llu B does not cover the pack-independent reserve",
                  (unsigned long long)budget);
    return fail(HMY_E_BUDGET_TOO_SMALL, "budget %llu B: even one layer per backward pack does not fit",
                (unsigned long long)budget);
  }
  *out = std::move(best);
  return HMY_OK;
}

}  // namespace hmy
