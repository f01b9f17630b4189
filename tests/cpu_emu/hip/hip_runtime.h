// Stand-in for <hip/hip_runtime.h> that lets g++ build the library's HIP sources for the HOST CPU:
// TEST INFRASTRUCTURE ONLY (tests/test_cpu_emulation.py).  The kernels run one work-group at a time,
// one OS thread per work-item, with barriers and the wave-level operations (shuffles, ballots, DPP,
// readlane) emulated for 64-lane waves; "device memory" is plain heap memory, so AddressSanitizer
// sees every access a kernel makes.  Nothing here is fast and nothing in the product path uses it.
#pragma once
#include <atomic>
#include <barrier>
#include <chrono>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <dlfcn.h>
#include <functional>
#include <map>
#include <memory>
#include <mutex>
#include <thread>
#include <vector>

// ---------------------------------------------------------------- language keywords
#define __global__
#define __device__
#define __host__
#define __forceinline__ inline
#define __noinline__ __attribute__((noinline))
#define __launch_bounds__(...)
#define __align__(n) alignas(n)

// ---------------------------------------------------------------- vector types
struct dim3 { unsigned x, y, z; dim3(unsigned a = 1, unsigned b = 1, unsigned c = 1) : x(a), y(b), z(c) {} };
struct alignas(16) float4 { float x, y, z, w; };
struct alignas(8) float2 { float x, y; };
struct alignas(16) ulonglong2 { unsigned long long x, y; };
struct alignas(16) double2 { double x, y; };
inline float4 make_float4(float a, float b, float c, float d) { return float4{a, b, c, d}; }
inline float2 make_float2(float a, float b) { return float2{a, b}; }

// ---------------------------------------------------------------- runtime stubs
typedef int hipError_t;
enum { hipSuccess = 0, hipErrorOutOfMemory = 2, hipErrorInvalidValue = 1 };
typedef void* hipStream_t;
typedef void* hipEvent_t;
enum hipMemcpyKind { hipMemcpyHostToDevice = 1, hipMemcpyDeviceToHost = 2, hipMemcpyDeviceToDevice = 3 };
enum { hipEventDisableTiming = 2, hipHostMallocMapped = 2, hipFuncAttributeMaxDynamicSharedMemorySize = 8 };
// device memory comes back holding garbage (0xBE bytes, or EMU_POISON: indices far out of range, floats near -0.37):
// whatever a kernel reads before it was written must not be able to steer an access
inline int emu_poison_byte() {
  static const int b = getenv("EMU_POISON") ? (int)strtol(getenv("EMU_POISON"), nullptr, 0) & 0xff : 0xBE;
  return b;
}
inline hipError_t hipMalloc(void** p, size_t n) {
  if (posix_memalign(p, 256, n ? n : 1) != 0) *p = nullptr;   // (hipMalloc returns 256-byte aligned memory)
  if (*p) memset(*p, emu_poison_byte(), n ? n : 1);
  return *p ? hipSuccess : hipErrorOutOfMemory;
}
template <class T> inline hipError_t hipMalloc(T** p, size_t n) { return hipMalloc((void**)p, n); }
inline hipError_t hipFree(void* p) { free(p); return hipSuccess; }
inline hipError_t hipHostMalloc(void** p, size_t n, unsigned = 0) { return hipMalloc(p, n); }
inline hipError_t hipHostFree(void* p) { free(p); return hipSuccess; }
inline hipError_t hipHostGetDevicePointer(void** d, void* h, unsigned) { *d = h; return hipSuccess; }
inline hipError_t hipMemcpyAsync(void* d, const void* s, size_t n, hipMemcpyKind, hipStream_t) { memcpy(d, s, n); return hipSuccess; }
inline hipError_t hipMemsetAsync(void* d, int v, size_t n, hipStream_t) { memset(d, v, n); return hipSuccess; }
inline hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
inline hipError_t hipGetLastError() { return hipSuccess; }
inline hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
inline hipError_t hipSetDevice(int) { return hipSuccess; }
inline hipError_t hipEventCreateWithFlags(hipEvent_t* e, unsigned) { *e = nullptr; return hipSuccess; }
inline hipError_t hipEventCreate(hipEvent_t* e) { *e = nullptr; return hipSuccess; }
inline hipError_t hipEventDestroy(hipEvent_t) { return hipSuccess; }
inline hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
inline hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
inline hipError_t hipEventElapsedTime(float* ms, hipEvent_t, hipEvent_t) { *ms = 0.0f; return hipSuccess; }
inline hipError_t hipFuncSetAttribute(const void*, int, int) { return hipSuccess; }
#define HIP_SYMBOL(x) ((const void*)&(x))
inline hipError_t hipGetSymbolAddress(void** p, const void* symbol) { *p = const_cast<void*>(symbol); return hipSuccess; }

// ---------------------------------------------------------------- SIMT emulation
namespace emu {
struct WorkGroup {
  int n_threads = 0, n_waves = 0;
  std::unique_ptr<std::barrier<>> wg_bar;
  std::vector<std::unique_ptr<std::barrier<>>> wave_bar;
  std::vector<std::unique_ptr<std::barrier<>>> row_bar;   // rows of 16 lanes: DPP operations that stay inside a row
  std::vector<uint64_t> xch;            // [n_waves][64] exchange slots of the wave operations
  std::vector<unsigned char> dyn;       // dynamic LDS of the running work-group
  std::vector<unsigned char> arena;     // static LDS of the running work-group, handed out per declaration
  std::map<int, size_t> arena_at;       // declaration -> offset
  size_t arena_used = 0;
  std::mutex arena_mu;
  std::vector<std::atomic<int>> at;     // per work-item: AT_*
  std::vector<const void*> where;       // per work-item: return address of the operation it waits in
  std::atomic<long long> ticks{0};      // bumped by every barrier passage
  void fresh() {                        // LDS of a new work-group: not zeros
    memset(arena.data(), 0xAB, arena.size());
    memset(dyn.data(), 0xAB, dyn.size());
    arena_at.clear(); arena_used = 0;
  }
};
struct Self {
  dim3 tid, bid, bdim, gdim;
  int lane = 0, wave = 0, flat = 0;
  WorkGroup* wg = nullptr;
};
// where every work-item currently is (0 running, 1 in a work-group barrier, 2 in a wave operation,
// 3 done with the work-group), for the watchdog's report when nothing moves any more
enum { AT_RUN = 0, AT_WG_BARRIER = 1, AT_WAVE_OP = 2, AT_DONE = 3 };
inline Self& self() { static thread_local Self s; return s; }
inline void wg_barrier() {
  Self& s = self();
  s.wg->where[s.flat] = __builtin_return_address(0);
  s.wg->at[s.flat] = AT_WG_BARRIER;
  s.wg->wg_bar->arrive_and_wait();
  s.wg->at[s.flat] = AT_RUN;
  s.wg->ticks++;
}
inline void wave_sync(Self& s, const void* ra, bool row_only = false) {
  s.wg->where[s.flat] = ra;
  s.wg->at[s.flat] = AT_WAVE_OP;
  if (row_only) s.wg->row_bar[s.flat >> 4]->arrive_and_wait();
  else s.wg->wave_bar[s.wave]->arrive_and_wait();
  s.wg->at[s.flat] = AT_RUN;
  s.wg->ticks++;
}
inline unsigned char* dyn_smem() { return self().wg->dyn.data(); }
template <class T> inline T* lds(int key, size_t align) {
  WorkGroup* wg = self().wg;
  std::lock_guard<std::mutex> lock(wg->arena_mu);
  auto it = wg->arena_at.find(key);
  if (it == wg->arena_at.end()) {
    const size_t at = (wg->arena_used + align - 1) / align * align;
    if (at + sizeof(T) > wg->arena.size()) { fprintf(stderr, "emu: static LDS over 64 KB\n"); abort(); }
    wg->arena_used = at + sizeof(T);
    it = wg->arena_at.emplace(key, at).first;
  }
  return (T*)(wg->arena.data() + it->second);
}

// value of `v` as held by lane `src` of the caller's wave.  All 64 lanes take part, or, with row_only
// (an exchange that stays inside rows of 16 lanes), all lanes of the caller's row: code that runs such
// operations with some rows of a wave switched off is legal on the GPU and has to work here too
template <class T> inline T from_lane(T v, int src, bool row_only = false) {
  static_assert(sizeof(T) <= 8, "payload");
  Self& s = self();
  uint64_t bits = 0;
  memcpy(&bits, &v, sizeof(T));
  uint64_t* slot = s.wg->xch.data() + (size_t)s.wave * 64;
  slot[s.lane] = bits;
  wave_sync(s, __builtin_return_address(0), row_only);
  const uint64_t r = slot[src & 63];
  wave_sync(s, __builtin_return_address(0), row_only);
  T out;
  memcpy(&out, &r, sizeof(T));
  return out;
}

// run `fn` once per work-item of a grid, one work-group after the other
inline void launch(dim3 grid, dim3 block, size_t smem, const std::function<void()>& fn) {
  const int nt = (int)(block.x * block.y * block.z);
  if (nt % 64 != 0 && nt > 64) { fprintf(stderr, "emu: block of %d threads\n", nt); abort(); }
  WorkGroup wg;
  wg.n_threads = nt; wg.n_waves = (nt + 63) / 64;
  wg.wg_bar = std::make_unique<std::barrier<>>(nt);
  for (int w = 0; w < wg.n_waves; ++w) {
    const int in_wave = std::min(64, nt - 64 * w);
    wg.wave_bar.push_back(std::make_unique<std::barrier<>>(in_wave));
  }
  for (int r = 0; r < (nt + 15) / 16; ++r) wg.row_bar.push_back(std::make_unique<std::barrier<>>(std::min(16, nt - 16 * r)));
  wg.xch.assign((size_t)wg.n_waves * 64, 0);
  wg.dyn.assign(smem + 64, 0);
  wg.arena.assign(64 * 1024 + 64, 0);
  wg.at = std::vector<std::atomic<int>>(nt);
  wg.where.assign(nt, nullptr);
  wg.fresh();
  // watchdog: a work-group in which nothing has moved for 20 s is stuck (a wave operation or a barrier
  // that not every work-item reaches): say where everybody is and give up
  std::atomic<bool> stop{false};
  std::thread dog([&]() {
    long long seen = -1; int idle = 0;
    while (!stop.load()) {
      std::this_thread::sleep_for(std::chrono::milliseconds(500));
      const long long now = wg.ticks.load();
      idle = now == seen ? idle + 1 : 0;
      seen = now;
      if (idle >= 40) {
        fprintf(stderr, "emu: work-group stuck (%d work-items):\n", nt);
        for (int w = 0; w < wg.n_waves; ++w) {
          int c[4] = {0, 0, 0, 0};
          for (int l = 0; l < 64 && w * 64 + l < nt; ++l) c[wg.at[w * 64 + l].load()]++;
          fprintf(stderr, "  wave %d: running %d, at work-group barrier %d, in wave operation %d, done %d;", w, c[0], c[1], c[2], c[3]);
          for (int l = 0; l < 64 && w * 64 + l < nt; l += 21)
          {
            Dl_info info;
            const void* a = wg.where[w * 64 + l];
            if (a && dladdr(a, &info) && info.dli_fbase)
              fprintf(stderr, " lane %d: state %d at +0x%zx", l, wg.at[w * 64 + l].load(),
                      (size_t)((const char*)a - (const char*)info.dli_fbase));
          }
          fprintf(stderr, "\n");
        }
        abort();
      }
    }
  });
  auto between = [&wg]() noexcept { wg.fresh(); };
  std::barrier<decltype(between)> next(nt, between);
  auto body = [&](int t) {
    Self& s = self();
    s.wg = &wg; s.bdim = block; s.gdim = grid;
    s.tid = dim3(t % block.x, (t / block.x) % block.y, t / (block.x * block.y));
    s.lane = t & 63; s.wave = t >> 6; s.flat = t;
    for (unsigned z = 0; z < grid.z; ++z)
      for (unsigned y = 0; y < grid.y; ++y)
        for (unsigned x = 0; x < grid.x; ++x) {
          s.bid = dim3(x, y, z);
          fn();
          wg.at[t] = AT_DONE;
          next.arrive_and_wait();        // the whole work-group is done before the next one starts
          wg.at[t] = AT_RUN;
          wg.ticks++;
        }
  };
  std::vector<std::thread> th;
  th.reserve(nt);
  for (int t = 1; t < nt; ++t) th.emplace_back(body, t);
  body(0);
  for (auto& x : th) x.join();
  stop = true;
  dog.join();
}
}  // namespace emu

#define threadIdx (emu::self().tid)
#define blockIdx (emu::self().bid)
#define blockDim (emu::self().bdim)
#define gridDim (emu::self().gdim)
#define hipLaunchKernelGGL(kernel, grid, block, smem, stream, ...) \
  emu::launch((grid), (block), (size_t)(smem), [&]() { kernel(__VA_ARGS__); })

inline void __syncthreads() { emu::wg_barrier(); }
inline void __threadfence() { std::atomic_thread_fence(std::memory_order_seq_cst); }
inline void __threadfence_system() { std::atomic_thread_fence(std::memory_order_seq_cst); }

// ---------------------------------------------------------------- wave operations
template <class T> inline T __shfl(T v, int lane) { return emu::from_lane(v, lane); }
template <class T> inline T __shfl_xor(T v, int mask) { return emu::from_lane(v, emu::self().lane ^ mask); }
template <class T> inline T __shfl_up(T v, int d) {
  const int l = emu::self().lane;
  const T o = emu::from_lane(v, l >= d ? l - d : l);
  return l >= d ? o : v;
}
inline unsigned long long __ballot(int pred) {
  emu::Self& s = emu::self();
  uint64_t* slot = s.wg->xch.data() + (size_t)s.wave * 64;
  slot[s.lane] = pred != 0 ? 1 : 0;
  emu::wave_sync(s, __builtin_return_address(0));
  const int n = std::min(64, s.wg->n_threads - 64 * s.wave);
  unsigned long long m = 0;
  for (int i = 0; i < n; ++i) m |= (unsigned long long)(slot[i] & 1) << i;
  emu::wave_sync(s, __builtin_return_address(0));
  return m;
}
inline int __builtin_amdgcn_readlane(int v, int lane) { return emu::from_lane(v, lane); }
// (on the GPU a scheduling fence only; here the lanes of a wave are threads and meet)
inline void __builtin_amdgcn_wave_barrier() { emu::wave_sync(emu::self(), __builtin_return_address(0)); }
// bits of a 64-bit lane mask (given as its two halves) set below the calling lane, plus `add`
inline unsigned __builtin_amdgcn_mbcnt_lo(unsigned m, unsigned add) {
  const int l = emu::self().lane;
  const unsigned below = l >= 32 ? 0xffffffffu : ((1u << l) - 1u);
  return (unsigned)__builtin_popcount(m & below) + add;
}
inline unsigned __builtin_amdgcn_mbcnt_hi(unsigned m, unsigned add) {
  const int l = emu::self().lane;
  const unsigned below = l <= 32 ? 0u : ((1u << (l - 32)) - 1u);
  return (unsigned)__builtin_popcount(m & below) + add;
}
// DPP controls of GFX9 (all lanes active, bank mask 0xf): quad_perm, row_shl/shr/ror, wave_shr:1,
// row_mirror, row_bcast15, row_bcast31; a lane without a source, or in a row that the row mask
// leaves out, keeps `old`
inline int __builtin_amdgcn_update_dpp(int old, int src, int ctrl, int row_mask, int bank_mask, bool bound_ctrl) {
  const int l = emu::self().lane, row = l >> 4, in = l & 15;
  int from = -1;
  if (ctrl >= 0x00 && ctrl <= 0xFF) from = (l & ~3) | ((ctrl >> (2 * (l & 3))) & 3);
  else if (ctrl >= 0x101 && ctrl <= 0x10F) { const int n = ctrl & 15; if (in + n <= 15) from = l + n; }
  else if (ctrl >= 0x111 && ctrl <= 0x11F) { const int n = ctrl & 15; if (in >= n) from = l - n; }
  else if (ctrl >= 0x121 && ctrl <= 0x12F) { const int n = ctrl & 15; from = (l & ~15) | ((in - n) & 15); }
  else if (ctrl == 0x138) { if (l >= 1) from = l - 1; }
  else if (ctrl == 0x130) { if (l <= 62) from = l + 1; }
  else if (ctrl == 0x140) from = (l & ~15) | (15 - in);
  else if (ctrl == 0x141) from = (l & ~7) | (7 - (l & 7));
  else if (ctrl == 0x142) { if (row >= 1) from = (row - 1) * 16 + 15; }
  else if (ctrl == 0x143) { if (row >= 2) from = 31; }
  else { fprintf(stderr, "emu: DPP control 0x%x not modelled\n", ctrl); abort(); }
  if (bank_mask != 0xf) { fprintf(stderr, "emu: DPP bank mask 0x%x not modelled\n", bank_mask); abort(); }
  const bool row_only = ctrl <= 0x12F || ctrl == 0x140 || ctrl == 0x141;
  const int got = emu::from_lane(src, from < 0 ? l : from, row_only);   // (every lane of the wave / row takes part)
  const bool row_on = (row_mask >> row) & 1;
  if (!row_on) return old;
  if (from < 0) return bound_ctrl ? 0 : old;
  return got;
}

// the older form: no old value (a lane without a source reads 0 with bound_ctrl, else is undefined: here 0)
inline int __builtin_amdgcn_mov_dpp(int src, int ctrl, int row_mask, int bank_mask, bool bound_ctrl) {
  return __builtin_amdgcn_update_dpp(0, src, ctrl, row_mask, bank_mask, bound_ctrl);
}

// ---------------------------------------------------------------- scalar intrinsics
inline int min(int a, int b) { return a < b ? a : b; }
inline int max(int a, int b) { return a > b ? a : b; }
inline unsigned min(unsigned a, unsigned b) { return a < b ? a : b; }
inline unsigned max(unsigned a, unsigned b) { return a > b ? a : b; }
inline long long min(long long a, long long b) { return a < b ? a : b; }
inline long long max(long long a, long long b) { return a > b ? a : b; }
inline unsigned long long min(unsigned long long a, unsigned long long b) { return a < b ? a : b; }
inline unsigned long long max(unsigned long long a, unsigned long long b) { return a > b ? a : b; }
inline float min(float a, float b) { return fminf(a, b); }
inline float max(float a, float b) { return fmaxf(a, b); }
inline double min(double a, double b) { return fmin(a, b); }
inline double max(double a, double b) { return fmax(a, b); }
inline int __popc(unsigned v) { return __builtin_popcount(v); }
inline int __popcll(unsigned long long v) { return __builtin_popcountll(v); }
inline int __ffs(int v) { return __builtin_ffs(v); }
inline int __float_as_int(float f) { int i; memcpy(&i, &f, 4); return i; }
inline unsigned __float_as_uint(float f) { unsigned i; memcpy(&i, &f, 4); return i; }
inline float __int_as_float(int i) { float f; memcpy(&f, &i, 4); return f; }
inline float __uint_as_float(unsigned i) { float f; memcpy(&f, &i, 4); return f; }
inline long long __double_as_longlong(double d) { long long i; memcpy(&i, &d, 8); return i; }
inline double __longlong_as_double(long long i) { double d; memcpy(&d, &i, 8); return d; }
inline float __expf(float x) { return expf(x); }
inline float __logf(float x) { return logf(x); }
inline float __builtin_amdgcn_exp2f(float x) { return exp2f(x); }
inline float __builtin_amdgcn_logf(float x) { return log2f(x); }            // (v_log_f32 is a base-2 logarithm)

// ---------------------------------------------------------------- atomics (device and LDS memory alike)
inline int atomicAdd(int* p, int v) { return __atomic_fetch_add(p, v, __ATOMIC_SEQ_CST); }
inline unsigned atomicAdd(unsigned* p, unsigned v) { return __atomic_fetch_add(p, v, __ATOMIC_SEQ_CST); }
inline unsigned long long atomicAdd(unsigned long long* p, unsigned long long v) { return __atomic_fetch_add(p, v, __ATOMIC_SEQ_CST); }
inline int atomicOr(int* p, int v) { return __atomic_fetch_or(p, v, __ATOMIC_SEQ_CST); }
template <class T> inline T emu_atomic_minmax(T* p, T v, bool is_min) {
  T cur = __atomic_load_n(p, __ATOMIC_SEQ_CST);
  while ((is_min ? v < cur : v > cur) &&
         !__atomic_compare_exchange_n(p, &cur, v, false, __ATOMIC_SEQ_CST, __ATOMIC_SEQ_CST)) {}
  return cur;
}
inline int atomicMin(int* p, int v) { return emu_atomic_minmax(p, v, true); }
inline int atomicMax(int* p, int v) { return emu_atomic_minmax(p, v, false); }
inline unsigned long long atomicMin(unsigned long long* p, unsigned long long v) { return emu_atomic_minmax(p, v, true); }
inline unsigned long long atomicMax(unsigned long long* p, unsigned long long v) { return emu_atomic_minmax(p, v, false); }
