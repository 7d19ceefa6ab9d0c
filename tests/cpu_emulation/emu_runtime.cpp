// Fiber-based CPU execution of one HIP workgroup at a time: one OS thread per wavefront, the 64
// lanes of a wavefront are ucontext fibers switched cooperatively at wave collectives and
// barriers.  AddressSanitizer is told about every stack switch.
#include <hip/hip_runtime.h>
#include <condition_variable>
#include <mutex>
#include <thread>
#include <vector>
#include <atomic>
#include <stdio.h>
#include <stdlib.h>
#include <sys/mman.h>

#if defined(__has_feature)
#if __has_feature(address_sanitizer)
#define EMU_ASAN 1
#endif
#endif
#ifdef EMU_ASAN
extern "C" void __sanitizer_start_switch_fiber(void **fake_stack_save, const void *bottom, size_t size);
extern "C" void __sanitizer_finish_switch_fiber(void *fake_stack_save, const void **bottom_old, size_t *size_old);
#endif

// minimal x86-64 context switch (callee-saved registers + stack pointer); no signal-mask syscalls
extern "C" void emu_switch(void **save_sp, void *new_sp);
asm(R"(
.text
.globl emu_switch
.type emu_switch,@function
emu_switch:
  pushq %rbp
  pushq %rbx
  pushq %r12
  pushq %r13
  pushq %r14
  pushq %r15
  movq %rsp, (%rdi)
  movq %rsi, %rsp
  popq %r15
  popq %r14
  popq %r13
  popq %r12
  popq %rbx
  popq %rbp
  ret
.size emu_switch,.-emu_switch
)");

#if defined(__has_feature)
#if __has_feature(thread_sanitizer)
#define EMU_TSAN 1
extern "C" void *__tsan_get_current_fiber(void);
extern "C" void *__tsan_create_fiber(unsigned flags);
extern "C" void __tsan_destroy_fiber(void *fiber);
extern "C" void __tsan_switch_to_fiber(void *fiber, unsigned flags);
#endif
#endif

namespace emu {
thread_local dim3 t_threadIdx;
dim3 g_blockIdx, g_blockDim, g_gridDim;

namespace {
constexpr int NW = 8, WL = 64;
constexpr size_t STACK = 512 * 1024;

enum State { RUNNABLE, AT_WAVE, AT_BLOCK, DONE };

struct Lane {
  void *sp = nullptr;
  char *stack = nullptr;
  State st = DONE;
  void *fake = nullptr;
  void *tsan = nullptr;
};

struct Wave {
  Lane lanes[WL];
  void *sched_sp = nullptr;
  void *sched_fake = nullptr;
  void *sched_tsan = nullptr;
  const void *sched_bottom = nullptr;
  size_t sched_size = 0;
  int cur = -1, nlanes = 0, id = 0;
  uint64_t slots[WL];
  float mfa[WL], mfb[WL];
};

Wave waves[NW];
thread_local Wave *t_wave = nullptr;
void *g_lds = nullptr;
const std::function<void()> *g_body = nullptr;

// block barrier among wave threads (spinning: at most eight threads take part)
std::atomic<int> b_alive{0}, b_arrived{0};
std::atomic<unsigned> b_gen{0};
std::mutex bm;
inline void spin_pause(int &n) { if (++n > 20000) { std::this_thread::yield(); n = 0; } else __builtin_ia32_pause(); }
void block_wait() {
  unsigned g;
  {
    std::lock_guard<std::mutex> l(bm);
    g = b_gen.load();
    if (b_arrived.load() + 1 >= b_alive.load()) { b_arrived = 0; b_gen = g + 1; return; }
    b_arrived = b_arrived.load() + 1;
  }
  int n = 0;
  while (b_gen.load(std::memory_order_acquire) == g) spin_pause(n);
}
void block_leave() {
  std::lock_guard<std::mutex> l(bm);
  b_alive = b_alive.load() - 1;
  if (b_alive.load() > 0 && b_arrived.load() >= b_alive.load()) { b_arrived = 0; b_gen = b_gen.load() + 1; }
}

// pool control (spinning)
std::atomic<unsigned> start_gen{0};
std::atomic<int> done_count{0};
std::atomic<bool> quit{false};
std::vector<std::thread> pool;

void to_scheduler(Wave *w, Lane *ln, bool dying) {
#ifdef EMU_ASAN
  __sanitizer_start_switch_fiber(dying ? nullptr : &ln->fake, w->sched_bottom, w->sched_size);
#endif
#ifdef EMU_TSAN
  __tsan_switch_to_fiber(w->sched_tsan, 0);
#endif
  emu_switch(&ln->sp, w->sched_sp);
#ifdef EMU_ASAN
  __sanitizer_finish_switch_fiber(ln->fake, &w->sched_bottom, &w->sched_size);
#endif
}

void lane_entry() {
  Wave *w = t_wave;
  Lane *ln = &w->lanes[w->cur];
#ifdef EMU_ASAN
  __sanitizer_finish_switch_fiber(nullptr, &w->sched_bottom, &w->sched_size);
#endif
  (*g_body)();
  ln->st = DONE;
  to_scheduler(w, ln, true);
  abort();  // never resumed
}

void yield(State why) {
  Wave *w = t_wave;
  Lane *ln = &w->lanes[w->cur];
  ln->st = why;
  to_scheduler(w, ln, false);
}

void run_wave(Wave *w) {
  t_wave = w;
  for (int l = 0; l < w->nlanes; ++l) {
    Lane &ln = w->lanes[l];
    if (!ln.stack) {
      ln.stack = (char *)mmap(nullptr, STACK, PROT_READ | PROT_WRITE, MAP_PRIVATE | MAP_ANONYMOUS | MAP_STACK, -1, 0);
      if (ln.stack == MAP_FAILED) abort();
    }
    {
      uintptr_t top = ((uintptr_t)ln.stack + STACK) & ~(uintptr_t)15;
      uint64_t *slot = (uint64_t *)(top - 16);  // 16-aligned: after `ret` the entry sees rsp = 8 mod 16
      slot[0] = (uint64_t)(uintptr_t)&lane_entry;
      slot[1] = 0;
      uint64_t *sp = slot - 6;
      for (int k = 0; k < 6; ++k) sp[k] = 0;
      ln.sp = sp;
    }
    ln.st = RUNNABLE;
    ln.fake = nullptr;
#ifdef EMU_TSAN
    ln.tsan = __tsan_create_fiber(0);
#endif
  }
#ifdef EMU_TSAN
  w->sched_tsan = __tsan_get_current_fiber();
#endif
  for (int l = w->nlanes; l < WL; ++l) w->lanes[l].st = DONE;
  for (;;) {
    bool ran = false;
    for (int l = 0; l < w->nlanes; ++l) {
      Lane &ln = w->lanes[l];
      if (ln.st != RUNNABLE) continue;
      ran = true;
      w->cur = l;
      t_threadIdx = dim3((unsigned)(w->id * WL + l), 0, 0);
#ifdef EMU_ASAN
      __sanitizer_start_switch_fiber(&w->sched_fake, ln.stack, STACK);
#endif
#ifdef EMU_TSAN
      __tsan_switch_to_fiber(ln.tsan, 0);
#endif
      emu_switch(&w->sched_sp, ln.sp);
#ifdef EMU_ASAN
      __sanitizer_finish_switch_fiber(w->sched_fake, nullptr, nullptr);
#endif
    }
    if (ran) continue;
    int nw = 0, nb = 0, nd = 0;
    for (int l = 0; l < w->nlanes; ++l) {
      State s = w->lanes[l].st;
      nw += s == AT_WAVE; nb += s == AT_BLOCK; nd += s == DONE;
    }
    if (nd == w->nlanes) {
#ifdef EMU_TSAN
      for (int l = 0; l < w->nlanes; ++l) { __tsan_destroy_fiber(w->lanes[l].tsan); w->lanes[l].tsan = nullptr; }
#endif
      break;
    }
    if (nw && nb) {
      fprintf(stderr, "emu: wave %d of block %u: %d lanes wait at a wave collective while %d wait at a barrier (divergent collective)\n",
              w->id, g_blockIdx.x, nw, nb);
      abort();
    }
    if (nb) block_wait();
    for (int l = 0; l < w->nlanes; ++l)
      if (w->lanes[l].st == AT_WAVE || w->lanes[l].st == AT_BLOCK) w->lanes[l].st = RUNNABLE;
  }
  block_leave();
}

void worker(int wid) {
  unsigned seen = 0;
  for (;;) {
    int n = 0;
    while (!quit.load() && start_gen.load(std::memory_order_acquire) == seen) spin_pause(n);
    if (quit.load()) return;
    seen = start_gen.load();
    if (waves[wid].nlanes > 0) run_wave(&waves[wid]);
    done_count.fetch_add(1, std::memory_order_release);
  }
}

void ensure_pool() {
  if (!pool.empty()) return;
  for (int t = 0; t < NW; ++t) { waves[t].id = t; pool.emplace_back(worker, t); }
  atexit([] {
    quit = true;
    for (auto &t : pool) t.join();
  });
}
}  // namespace

// Host-only regions: memory a kernel must never touch (host structs of the C ABI, the host copies of
// the table descriptors).  With AddressSanitizer they are poisoned for the duration of every launch, so
// a kernel that dereferences a host pointer -- which works on the CPU and faults on a GPU -- is reported.
#if defined(__has_feature)
#if __has_feature(address_sanitizer)
#define EMU_ASAN 1
extern "C" void __asan_poison_memory_region(void const volatile *addr, size_t size);
extern "C" void __asan_unpoison_memory_region(void const volatile *addr, size_t size);
#endif
#endif
namespace {
struct HostOnly { const void *p; size_t n; };
std::vector<HostOnly> host_only_regions;
void poison_host_only(bool on) {
#ifdef EMU_ASAN
  for (const HostOnly &r : host_only_regions) {
    if (on) __asan_poison_memory_region(r.p, r.n); else __asan_unpoison_memory_region(r.p, r.n);
  }
#else
  (void)on;
#endif
}
}  // namespace
void host_only(const void *p, size_t n) { host_only_regions.push_back({p, n}); }
void host_only_release(const void *p) {
  for (size_t i = 0; i < host_only_regions.size(); ++i)
    if (host_only_regions[i].p == p) { host_only_regions.erase(host_only_regions.begin() + i); return; }
}

void launch(dim3 grid, dim3 block, size_t lds, const char *name, const std::function<void()> &body) {
  ensure_pool();
  if (block.x > NW * WL || block.y != 1 || block.z != 1 || grid.x == 0 || grid.y == 0) {
    fprintf(stderr, "emu: bad launch %s grid %u,%u block %u\n", name, grid.x, grid.y, block.x);
    abort();
  }
  if (getenv("EMU_TRACE")) fprintf(stderr, "emu: launch %s grid (%u,%u) block %u lds %zu\n", name, grid.x, grid.y, block.x, lds);
  g_gridDim = grid; g_blockDim = block;
  g_lds = lds ? malloc(lds) : nullptr;   // exact size: ASan sees dynamic-LDS overruns
  if (g_lds) memset(g_lds, 0x7F, lds);   // defined garbage (NaN pattern): uninitialised-read hunts target global memory
  // EMU_REVERSE runs the workgroups of a launch last to first: results must not depend on the order
  static const bool reverse = getenv("EMU_REVERSE") != nullptr;
  // EMU_SHUFFLE=<seed> runs them in a seeded random order over BOTH grid dimensions, so that the
  // workgroups of different tables of a batched launch are interleaved
  static const char *shuffle = getenv("EMU_SHUFFLE");
  std::vector<unsigned> order((size_t)grid.x * grid.y);
  for (size_t i = 0; i < order.size(); ++i) order[i] = (unsigned)i;
  if (shuffle) {
    static uint64_t rs = 0x9E3779B97F4A7C15ull ^ strtoull(shuffle, nullptr, 0);
    for (size_t i = order.size(); i > 1; --i) {
      rs ^= rs << 13; rs ^= rs >> 7; rs ^= rs << 17;
      std::swap(order[i - 1], order[(size_t)(rs % i)]);
    }
  }
  poison_host_only(true);
  for (size_t oi = 0; oi < order.size(); ++oi) {
    {
      const unsigned by = order[oi] / grid.x, bi = order[oi] % grid.x;
      const unsigned bx = reverse ? grid.x - 1 - bi : bi;
      g_blockIdx = dim3(bx, by, 0);
      int nwaves = 0;
      for (int w = 0; w < NW; ++w) {
        int n = (int)block.x - WL * w;
        waves[w].nlanes = n < 0 ? 0 : (n > WL ? WL : n);
        nwaves += waves[w].nlanes > 0;
      }
      b_alive = nwaves; b_arrived = 0;
      g_body = &body; done_count = 0;
      start_gen.fetch_add(1, std::memory_order_release);
      { int n = 0; while (done_count.load(std::memory_order_acquire) != NW) spin_pause(n); }
    }
  }
  poison_host_only(false);
  free(g_lds);
  g_lds = nullptr;
}

void syncthreads() { yield(AT_BLOCK); }
void *dyn_lds() { return g_lds; }

uint64_t wave_exchange(uint64_t v, int src_lane) {
  Wave *w = t_wave;
  const int lane = w->cur;
  w->slots[lane] = v;
  yield(AT_WAVE);
  uint64_t r = v;
  if (src_lane == -2) {
    for (int l = 0; l < WL; ++l) if (w->lanes[l].st != DONE) { r = w->slots[l]; break; }
  } else if (src_lane >= 0 && src_lane < WL) {
    r = w->slots[src_lane];
  }
  yield(AT_WAVE);
  return r;
}

uint64_t wave_ballot(bool pred) {
  Wave *w = t_wave;
  const int lane = w->cur;
  w->slots[lane] = pred ? 1 : 0;
  yield(AT_WAVE);
  uint64_t m = 0;
  for (int l = 0; l < WL; ++l) if (w->lanes[l].st != DONE && w->slots[l]) m |= (1ull << l);
  yield(AT_WAVE);
  return m;
}

void wave_mfma_16x16x4(float a, float b, float *c4) {
  Wave *w = t_wave;
  const int lane = w->cur;
  w->mfa[lane] = a; w->mfb[lane] = b;
  yield(AT_WAVE);
  const int n = lane & 15;
  for (int v = 0; v < 4; ++v) {
    const int m = 4 * (lane >> 4) + v;
    float s = c4[v];
    for (int k = 0; k < 4; ++k) s += w->mfa[k * 16 + m] * w->mfb[k * 16 + n];
    c4[v] = s;
  }
  yield(AT_WAVE);
}
}  // namespace emu
