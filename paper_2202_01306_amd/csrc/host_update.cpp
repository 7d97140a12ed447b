// The Weight Update task on the host CPU (Harmony paper, Section 4.4: the Runtime can
// place the update task on the CPU instead of the GPU).  Optimizer state and weights then
// never cross the host link: the backward task exports the pack's gradient to the pinned
// host array, and this file applies Adam to the pinned host arrays in place, chunk by chunk,
// as the chunks arrive.
//
// One dispatcher thread takes jobs in submission order, waits until the job's gradient has
// arrived (a callback of the engine's: it waits for the HIP event of that chunk's
// device->host copy; this file itself is plain host C++) and runs the update over a pool of
// worker threads.  The arithmetic is the same as the device kernel's (fp32; bias corrections passed
// in as reciprocals; bf16 weight = round-to-nearest-even of the fp32 master).  The inner
// loop is plain C++ compiled three times (AVX-512, AVX2+FMA, baseline) and picked at run
// time, because the library is built on one machine and runs on another.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <condition_variable>
#include <cstring>
#include <deque>
#include <functional>
#include <mutex>
#include <thread>

#include "hmy_internal.h"

namespace hmy {

namespace {

inline __attribute__((always_inline)) uint16_t bf16_rne(float x) {
  uint32_t u;
  std::memcpy(&u, &x, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return uint16_t((u >> 16) | 0x40);   // NaN stays NaN
  return uint16_t((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

template <bool MIXED>
inline __attribute__((always_inline)) void adam_span(const HostAdamJob &a, uint64_t lo, uint64_t hi) {
  const float *__restrict g = a.grad;
  float *__restrict w = MIXED ? a.master : static_cast<float *>(a.weights);
  float *__restrict m = a.m;
  float *__restrict v = a.v;
  uint16_t *__restrict w16 = MIXED ? static_cast<uint16_t *>(a.weights) : nullptr;
  const float lr = a.lr, b1 = a.b1, b2 = a.b2, eps = a.eps, c1 = a.inv_bc1, c2 = a.inv_bc2;
  const float o1 = 1.f - b1, o2 = 1.f - b2;
  for (uint64_t i = lo; i < hi; ++i) {
    const float gi = g[i];
    const float mm = b1 * m[i] + o1 * gi;
    const float vv = b2 * v[i] + o2 * gi * gi;
    const float wi = w[i] - lr * (mm * c1) / (__builtin_sqrtf(vv * c2) + eps);
    m[i] = mm;
    v[i] = vv;
    w[i] = wi;
    if (MIXED) w16[i] = bf16_rne(wi);
  }
}

__attribute__((target("avx512f,avx512bw,avx512vl,avx512dq,fma"))) void span_avx512(const HostAdamJob &a, uint64_t lo,
                                                                                   uint64_t hi) {
  if (a.master) adam_span<true>(a, lo, hi);
  else adam_span<false>(a, lo, hi);
}
__attribute__((target("avx2,fma"))) void span_avx2(const HostAdamJob &a, uint64_t lo, uint64_t hi) {
  if (a.master) adam_span<true>(a, lo, hi);
  else adam_span<false>(a, lo, hi);
}
void span_base(const HostAdamJob &a, uint64_t lo, uint64_t hi) {
  if (a.master) adam_span<true>(a, lo, hi);
  else adam_span<false>(a, lo, hi);
}

using SpanFn = void (*)(const HostAdamJob &, uint64_t, uint64_t);
SpanFn pick_span() {
  __builtin_cpu_init();
  if (__builtin_cpu_supports("avx512f") && __builtin_cpu_supports("avx512bw") && __builtin_cpu_supports("avx512vl") &&
      __builtin_cpu_supports("avx512dq"))
    return span_avx512;
  if (__builtin_cpu_supports("avx2") && __builtin_cpu_supports("fma")) return span_avx2;
  return span_base;
}

}  // namespace

HostAdamJob make_host_adam_job(void *ready, const float *grad, float *master, float *m, float *v, void *weights,
                               uint64_t n, const hmy_adam &hp) {
  HostAdamJob j;
  j.ready = ready;
  j.grad = grad;
  j.master = master;
  j.m = m;
  j.v = v;
  j.weights = weights;
  j.n = n;
  j.lr = hp.lr;
  j.b1 = hp.beta1;
  j.b2 = hp.beta2;
  j.eps = hp.eps;
  // bias corrections exactly as the device launcher computes them
  j.inv_bc1 = float(1.0 / (1.0 - std::pow(double(hp.beta1), double(hp.step))));
  j.inv_bc2 = float(1.0 / (1.0 - std::pow(double(hp.beta2), double(hp.step))));
  return j;
}

int default_host_threads() {
  // a GPU machine gives a process 16 cores per GPU whatever the machine has
  int nt = int(std::min(16u, std::max(1u, std::thread::hardware_concurrency())));
  if (const char *e = std::getenv("HMY_HOST_THREADS")) nt = std::max(1, std::min(256, std::atoi(e)));
  return nt;
}

struct HostUpdater::Impl {
  HostUpdater::Hook thread_init = nullptr, wait_ready = nullptr;
  void *hook_arg = nullptr;
  int nthreads = 1;
  SpanFn span = span_base;
  // pool: workers 1..nthreads-1 wait for a new generation; the dispatcher is worker 0
  std::vector<std::thread> workers;
  std::mutex pool_mu;
  std::condition_variable pool_work, pool_done;
  uint64_t generation = 0;
  int pending = 0;
  bool pool_stop = false;
  HostAdamJob cur{};
  // job queue
  std::thread dispatcher;
  std::mutex q_mu;
  std::condition_variable q_work, q_idle;
  std::deque<HostAdamJob> queue;
  bool busy = false, q_stop = false;
  int error = HMY_OK;

  void part(int tid) const {
    // contiguous ranges, 64-element aligned so that no two threads share a cache line of any array
    const uint64_t per = ((cur.n + nthreads - 1) / nthreads + 63) & ~uint64_t(63);
    const uint64_t lo = std::min<uint64_t>(cur.n, per * tid), hi = std::min<uint64_t>(cur.n, lo + per);
    if (hi > lo) span(cur, lo, hi);
  }
  void worker(int tid) {
    uint64_t seen = 0;
    for (;;) {
      {
        std::unique_lock<std::mutex> lk(pool_mu);
        pool_work.wait(lk, [&] { return pool_stop || generation != seen; });
        if (pool_stop) return;
        seen = generation;
      }
      part(tid);
      std::lock_guard<std::mutex> lk(pool_mu);
      if (--pending == 0) pool_done.notify_one();
    }
  }
  void run_job(const HostAdamJob &job) {
    {
      std::lock_guard<std::mutex> lk(pool_mu);
      cur = job;
      pending = nthreads - 1;
      ++generation;
    }
    pool_work.notify_all();
    part(0);
    std::unique_lock<std::mutex> lk(pool_mu);
    pool_done.wait(lk, [&] { return pending == 0; });
  }
  void dispatch() {
    if (thread_init) (void)thread_init(hook_arg, nullptr);
    for (;;) {
      HostAdamJob job;
      {
        std::unique_lock<std::mutex> lk(q_mu);
        q_work.wait(lk, [&] { return q_stop || !queue.empty(); });
        if (queue.empty()) return;   // stop requested and nothing left
        job = queue.front();
        queue.pop_front();
        busy = true;
      }
      int rc = HMY_OK;
      if (job.ready && wait_ready) rc = wait_ready(hook_arg, job.ready);
      if (rc == HMY_OK) run_job(job);
      {
        std::lock_guard<std::mutex> lk(q_mu);
        if (rc != HMY_OK && error == HMY_OK) error = rc;
        busy = false;
        if (queue.empty()) q_idle.notify_all();
      }
    }
  }
};

HostUpdater::HostUpdater(int nthreads, Hook thread_init, Hook wait_ready, void *hook_arg) : p(new Impl) {
  p->thread_init = thread_init;
  p->wait_ready = wait_ready;
  p->hook_arg = hook_arg;
  p->nthreads = std::max(1, nthreads);
  p->span = pick_span();
  for (int t = 1; t < p->nthreads; ++t) p->workers.emplace_back([this, t] { p->worker(t); });
  p->dispatcher = std::thread([this] { p->dispatch(); });
}

HostUpdater::~HostUpdater() {
  {
    std::lock_guard<std::mutex> lk(p->q_mu);
    p->q_stop = true;
  }
  p->q_work.notify_all();
  if (p->dispatcher.joinable()) p->dispatcher.join();
  {
    std::lock_guard<std::mutex> lk(p->pool_mu);
    p->pool_stop = true;
  }
  p->pool_work.notify_all();
  for (auto &w : p->workers) w.join();
  delete p;
}

void HostUpdater::submit(const HostAdamJob &job) {
  if (!job.n) return;
  {
    std::lock_guard<std::mutex> lk(p->q_mu);
    p->queue.push_back(job);
  }
  p->q_work.notify_one();
}

int HostUpdater::drain() {
  std::unique_lock<std::mutex> lk(p->q_mu);
  p->q_idle.wait(lk, [&] { return p->queue.empty() && !p->busy; });
  const int e = p->error;
  p->error = HMY_OK;
  return e;
}

int HostUpdater::threads() const { return p->nthreads; }

}  // namespace hmy
