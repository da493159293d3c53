// Kernel launches with optional per-launch timing.
//
// OSEQ_LAUNCH(kernel, grid, block, lds_bytes, stream, args...) is hipLaunchKernelGGL, except while the calling thread
// has a launch timer installed: then the launch carries a start and a stop event (hipExtLaunchKernel), which take
// their time stamps from the dispatch itself.  Unlike a pair of hipEventRecord calls around the launch this adds no
// packets to the queue, so the elapsed time is the kernel's own duration (what a kernel trace reports).
#pragma once
#include <hip/hip_runtime.h>

namespace oseq {

struct LaunchTimer {
  bool on = false;
  hipEvent_t (*next)(void* ctx) = nullptr;  // hands out events; consecutive pairs are (start, stop) of one launch
  void* ctx = nullptr;
};
extern thread_local LaunchTimer g_launch_timer;

}  // namespace oseq

#if defined(__HIPCC__)  // the launch side: translation units with kernels
#include <hip/hip_ext.h>

#include <tuple>
#include <utility>

namespace oseq {

template <typename... KArgs, size_t... I>
inline void launch_timed_impl(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t st, hipEvent_t e0,
                              hipEvent_t e1, std::tuple<KArgs...>& vals, std::index_sequence<I...>) {
  void* ptrs[] = {static_cast<void*>(&std::get<I>(vals))...};
  (void)hipExtLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds, st, e0, e1, 0);
}

// the arguments are converted to the kernel's exact parameter types, as the triple-chevron launch would do
template <typename... KArgs, typename... Args>
inline void launch_timed(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t st, hipEvent_t e0,
                         hipEvent_t e1, Args&&... args) {
  static_assert(sizeof...(KArgs) == sizeof...(Args), "argument count does not match the kernel");
  std::tuple<KArgs...> vals{static_cast<KArgs>(args)...};
  launch_timed_impl(kernel, grid, block, lds, st, e0, e1, vals, std::index_sequence_for<KArgs...>{});
}

}  // namespace oseq

#define OSEQ_LAUNCH(kernel, grid, block, lds, st, ...)                                                    \
  do {                                                                                                    \
    ::oseq::LaunchTimer& lt_ = ::oseq::g_launch_timer;                                                    \
    hipEvent_t e0_ = nullptr, e1_ = nullptr;                                                              \
    if (lt_.on && (e0_ = lt_.next(lt_.ctx)) && (e1_ = lt_.next(lt_.ctx)))                                 \
      ::oseq::launch_timed(kernel, grid, block, lds, st, e0_, e1_, __VA_ARGS__);                          \
    else                                                                                                  \
      hipLaunchKernelGGL(kernel, grid, block, lds, st, __VA_ARGS__);                                      \
  } while (0)
#endif
