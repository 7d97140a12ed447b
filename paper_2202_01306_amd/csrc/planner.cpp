// Pack planner: analytic layer profile, HBM arena layout and balanced-time
// packing (the paper's Algorithm 2, Section 4.3.1) under the HBM budget.
//
// Memory model.  The runtime keeps kSlots = 3 weight slots (prefetch distance 1,
// Section 4.4: the pack being computed, the next one arriving, and the previous
// one still draining through its update and write-back), one activation workspace
// for the backward pack in flight, and a pack-independent reserve (resident
// boundary activations, checkpoint rings, gradient scratch, the optimizer ring).
// A layer's footprint for the packing is therefore
//   forward : kSlots * E * p                   (E bytes per weight, p parameters)
//   backward: kSlots * (E + 4) * p + act       (weights + fp32 gradients per slot; activations once)
// and the capacity is the budget minus the reserve.  Times are flop counts of
// one microbatch (integers, so the balanced split has exact ties).
#include <algorithm>
#include <cstring>

#include "hmy_internal.h"

namespace hmy {

BlockActs block_acts(const hmy_model_spec &s, int micro_batch) {
  const uint64_t E = s.precision == HMY_PREC_BF16 ? 2 : 4;
  const uint64_t T = uint64_t(micro_batch) * s.seq_len, d = s.d_model, f = s.d_ffn, H = s.n_heads;
  BlockActs b;
  uint64_t off = 0;
  auto take = [&](uint64_t bytes) { uint64_t o = off; off += a256(bytes); return o; };
  b.x_in = take(T * d * E);
  b.a = take(T * d * E);
  b.qkv = take(3 * T * d * E);
  b.o = take(T * d * E);
  b.x_mid = take(T * d * E);
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
  h.x_in = take(T * d * E);
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

Reserved reserved_layout(const Model &m, int n_micro, int micro_batch) {
  const hmy_model_spec &s = m.spec;
  const uint64_t E = m.elem_bytes();
  const uint64_t T = uint64_t(micro_batch) * s.seq_len, d = s.d_model, f = s.d_ffn, H = s.n_heads;
  Reserved r;
  uint64_t off = 0;
  auto take = [&](uint64_t bytes) { uint64_t o = off; off += a256(bytes); return o; };
  r.x_bytes = a256(T * d * E);
  r.X = take(uint64_t(n_micro) * r.x_bytes);
  r.inring = take(kInRing * r.x_bytes);
  r.outring = take(kOutRing * r.x_bytes);
  r.gbig = take(T * std::max<uint64_t>(f, 3 * d) * E);
  r.gsmall = take(T * d * E);
  r.delta = take(T * H * 4);
  r.ids = take(uint64_t(n_micro) * T * 4);
  r.targets = take(uint64_t(n_micro) * T * 4);
  r.misc = take(4096);
  r.ln_ws = take(uint64_t(kLnBlocks) * 2 * d * 4);
  uint64_t maxp = 0;
  for (int l = 0; l < m.R; ++l) maxp = std::max(maxp, m.params_in(l, l + 1));
  r.k_chunk_params = std::min<uint64_t>(kKChunkMax, maxp);
  r.karr_bytes = a256(r.k_chunk_params * 4);
  r.kring = take(uint64_t(kKRing) * m.k_arrays() * r.karr_bytes);
  r.size = off;
  return r;
}

void layer_profile(const Model &m, int n_micro, int micro_batch, std::vector<hmy_layer_profile> *out) {
  (void)n_micro;
  const hmy_model_spec &s = m.spec;
  const int64_t T = int64_t(micro_batch) * s.seq_len, d = s.d_model, f = s.d_ffn, V = s.vocab;
  const uint64_t E = m.elem_bytes();
  out->assign(m.R, hmy_layer_profile{});
  const uint64_t act_block = block_acts(s, micro_batch).size;
  const uint64_t act_head = head_acts(s, micro_batch).size;
  for (int l = 0; l < m.R; ++l) {
    hmy_layer_profile &p = (*out)[l];
    p.params = m.params_in(l, l + 1);
    if (l == 0) {
      p.t_fwd = T * d;
      p.act_bwd = 0;
    } else if (l <= s.n_blocks) {
      p.t_fwd = T * (8 * d * d + 4 * d * f + (s.causal ? 2 : 4) * int64_t(s.seq_len) * d);
      p.act_bwd = act_block;
    } else {
      p.t_fwd = 2 * T * d * V;
      p.act_bwd = act_head;
    }
    p.t_bwd = 3 * p.t_fwd;
    p.mem_fwd = kSlots * E * p.params;
    p.mem_bwd = kSlots * (E + 4) * p.params + p.act_bwd;
  }
}

uint64_t pack_state_fwd(const Model &m, Pack p) { return a256(m.elem_bytes() * m.params_in(p.a, p.e)); }
uint64_t pack_state_bwd(const Model &m, Pack p) {
  return a256(m.elem_bytes() * m.params_in(p.a, p.e)) + a256(4 * m.params_in(p.a, p.e));
}

Arena arena_layout(const Model &m, const Packs &p, int n_micro, int micro_batch) {
  Arena a;
  a.res = reserved_layout(m, n_micro, micro_batch);
  std::vector<hmy_layer_profile> prof;
  layer_profile(m, n_micro, micro_batch, &prof);
  a.slot_bytes = 0;
  a.act_bytes = 0;
  for (const Pack &q : p.fwd) a.slot_bytes = std::max(a.slot_bytes, pack_state_fwd(m, q));
  for (const Pack &q : p.bwd) {
    a.slot_bytes = std::max(a.slot_bytes, pack_state_bwd(m, q));
    uint64_t act = 0;
    for (int l = q.a; l < q.e; ++l) act += prof[l].act_bwd;
    a.act_bytes = std::max(a.act_bytes, act);
  }
  for (int i = 0; i < kSlots; ++i) a.slot_off[i] = a.res.size + uint64_t(i) * a.slot_bytes;
  a.act_off = a.res.size + uint64_t(kSlots) * a.slot_bytes;
  a.total = a.act_off + a.act_bytes;
  return a;
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
  Packs p;
  p.resident_state = s->resident_state;
  p.order = s->order;
  p.update_site = s->update_site;
  p.gradients = s->gradients;
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

// Runtime estimate of one iteration for a packing (the role of the paper's Runtime
// Estimator, Section 4.3.1, reduced to what decides the pack count on one GPU): an
// event-driven walk of the task list over three resources -- the compute stream, the
// host->device link and the device->host link -- in integer nanoseconds.  Compute
// time of a visit = n_micro * sum of its layers' flops / rate; each visit's weights
// are requested when the previous visit starts computing and its slot is free; a
// backward visit's update moves its optimizer state in and (state, weights,
// gradients) out after its compute ends.  Checkpoint traffic is ignored (small).
uint64_t estimate_iteration_ns(const Model &m, const std::vector<hmy_layer_profile> &prof, const Packs &p, int n_micro,
                               uint64_t link_MBps, uint64_t compute_GFLOPs) {
  const uint64_t E = m.elem_bytes(), kB = 4 * uint64_t(m.k_arrays());
  auto t_bytes = [&](uint64_t bytes) { return (bytes * 1000 + link_MBps - 1) / link_MBps; };
  auto t_flops = [&](uint64_t flops) { return (flops + compute_GFLOPs - 1) / compute_GFLOPs; };
  // with the update on the host only the gradient crosses the link, and the CPU threads (about 6 parameters
  // per nanosecond on the machines measured) are one more queue
  const bool host = p.update_site == HMY_UPDATE_ON_HOST;
  constexpr uint64_t kHostParamsPerNs = 6;
  struct V { bool bwd; uint64_t comp, w, kin, out, cpu; };
  std::vector<V> vs;
  for (const Pack &q : p.fwd) {
    uint64_t fl = 0;
    for (int l = q.a; l < q.e; ++l) fl += uint64_t(prof[l].t_fwd);
    vs.push_back({false, t_flops(fl * n_micro), t_bytes(E * m.params_in(q.a, q.e)), 0, 0, 0});
  }
  for (int k = int(p.bwd.size()) - 1; k >= 0; --k) {
    const Pack &q = p.bwd[k];
    uint64_t fl = 0;
    for (int l = q.a; l < q.e; ++l) fl += uint64_t(prof[l].t_bwd);
    const uint64_t P = m.params_in(q.a, q.e);
    if (host) vs.push_back({true, t_flops(fl * n_micro), t_bytes(E * P), 0, t_bytes(4 * P), P / kHostParamsPerNs});
    else vs.push_back({true, t_flops(fl * n_micro), t_bytes(E * P), t_bytes(kB * P), t_bytes((kB + E + 4) * P), 0});
  }
  uint64_t h2d_free = 0, d2h_free = 0, comp_free = 0, cpu_free = 0, slot_free[kSlots] = {};
  std::vector<uint64_t> w_ready(vs.size() + 1, 0);
  w_ready[0] = vs[0].w;
  h2d_free = w_ready[0];
  for (size_t v = 0; v < vs.size(); ++v) {
    const uint64_t comp_start = std::max(comp_free, w_ready[v]);
    if (v + 1 < vs.size()) {
      const uint64_t s = std::max(std::max(comp_start, slot_free[(v + 1) % kSlots]), h2d_free);
      w_ready[v + 1] = s + vs[v + 1].w;
      h2d_free = w_ready[v + 1];
    }
    const uint64_t comp_end = comp_start + vs[v].comp;
    comp_free = comp_end;
    if (!vs[v].bwd) {
      slot_free[v % kSlots] = comp_end;
    } else {
      uint64_t kin_end = comp_end;
      if (!host) {
        kin_end = std::max(comp_end, h2d_free) + vs[v].kin;
        h2d_free = kin_end;
      }
      const uint64_t out_end = std::max(std::max(comp_end, d2h_free) + vs[v].out, kin_end);
      d2h_free = out_end;
      slot_free[v % kSlots] = out_end;
      if (host) cpu_free = std::max(cpu_free, out_end) + vs[v].cpu;
    }
  }
  return std::max(comp_free, std::max(d2h_free, cpu_free));
}

int plan_packs(const Model &m, const hmy_budget &b, int n_micro, int micro_batch, Packs *out) {
  const uint64_t budget = b.hbm_budget_bytes;
  const uint64_t link = b.host_link_MBps ? b.host_link_MBps : 40000, rate = b.compute_GFLOPs ? b.compute_GFLOPs : 420000;
  std::vector<hmy_layer_profile> prof;
  layer_profile(m, n_micro, micro_batch, &prof);
  if (b.update_site != HMY_UPDATE_ON_DEVICE && b.update_site != HMY_UPDATE_ON_HOST)
    return fail(HMY_E_INVALID, "budget: unknown update site %u", b.update_site);
  const Reserved res = reserved_layout(m, n_micro, micro_batch);
  if (budget <= res.size)
    return fail(HMY_E_BUDGET_TOO_SMALL, "budget %llu B does not cover the pack-independent reserve %llu B",
                (unsigned long long)budget, (unsigned long long)res.size);
  std::vector<int64_t> tb(m.R);
  std::vector<uint64_t> mb(m.R);
  for (int l = 0; l < m.R; ++l) {
    tb[l] = prof[l].t_bwd;
    mb[l] = prof[l].mem_bwd;
  }
  auto arena_fits = [&](const std::vector<Pack> &bwd) {
    Packs q;
    q.bwd = bwd;
    return arena_layout(m, q, n_micro, micro_batch).total <= budget;
  };
  auto always = [](const std::vector<Pack> &) { return true; };
  // Candidates: the first feasible pack count of Algorithm 2 (largest packs), then up to
  // max_extra_packs further feasible pack counts; as in Algorithm 1 the configuration with
  // the smallest estimated iteration time wins (ties: the earlier candidate).  When the
  // search is on, each balanced packing is also tried in three reshaped forms that the
  // balanced split cannot produce and the estimate can tell apart:
  //   taper : the first backward pack [0, e) becomes [0,1), [1,2), [2,e) -- the update of
  //           the pack visited last cannot hide behind any compute, so it should be small,
  //           and so should the one before it, which hides behind that short visit;
  //   merge : the last two backward packs become one (if the arena still fits) -- the last
  //           pack is not recomputed, and its layers drop out of the forward pass;
  //   both.
  bool have = false;
  uint64_t best_ns = 0;
  Packs best;
  int rc_fwd = HMY_OK;
  auto consider = [&](const std::vector<Pack> &bwd) {
    Packs p;
    p.bwd = bwd;
    p.update_site = int(b.update_site);
    // forward packs over the layers before the last backward pack; they share the
    // weight slots sized by the backward packing
    const int RF = p.bwd.back().a;
    Packs only_b;
    only_b.bwd = p.bwd;
    const uint64_t slot = arena_layout(m, only_b, n_micro, micro_batch).slot_bytes;
    std::vector<int64_t> tf(RF);
    std::vector<uint64_t> mf(RF);
    for (int l = 0; l < RF; ++l) {
      tf[l] = prof[l].t_fwd;
      mf[l] = prof[l].mem_fwd;
    }
    if (!balanced_time_packing(tf, mf, uint64_t(kSlots) * slot, 0, always, &p.fwd)) {
      rc_fwd = HMY_E_BUDGET_TOO_SMALL;
      return;
    }
    auto offer = [&](const Packs &q) {
      const uint64_t ns = estimate_iteration_ns(m, prof, q, n_micro, link, rate);
      if (!have || ns < best_ns) {
        have = true;
        best_ns = ns;
        best = q;
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
        if (mem > uint64_t(kSlots) * slot) ok = false;
        q.fwd.push_back({a, e});
        a = e;
      }
      if (ok) offer(q);
    }
  };
  auto taper = [](std::vector<Pack> v) {
    const int e = v.front().e;
    if (e < 2) return v;
    std::vector<Pack> head = {{0, 1}, {1, 2}};
    if (e > 2) head.push_back({2, e});
    else head.back().e = e;
    v.erase(v.begin());
    v.insert(v.begin(), head.begin(), head.end());
    return v;
  };
  int S_start = 1;
  for (uint32_t tries = 0; tries <= b.max_extra_packs; ++tries) {
    std::vector<Pack> bwd;
    int S_used = 0;
    // backward packs first (Algorithm 1, line "backward packing")
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
    if (rc_fwd) return fail(HMY_E_BUDGET_TOO_SMALL, "forward packing failed (internal)");
    if (S_used > m.R) break;   // that was the one-layer-per-pack fallback
    S_start = S_used + 1;
  }
  if (!have)
    return fail(HMY_E_BUDGET_TOO_SMALL, "budget %llu B: even one layer per backward pack does not fit",
                (unsigned long long)budget);
  *out = std::move(best);
  return HMY_OK;
}

}  // namespace hmy
