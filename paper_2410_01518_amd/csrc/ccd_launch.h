// Every kernel of libinfinipot is launched through ccd::launch.
//
// Ordinarily that is a plain launch.  While the per-kernel timing of the library is switched on (ccd_profile_enable, a
// bench aid) and a timed stage is open, the launch carries the stage's two events: the runtime then fills them with the
// begin and end time stamps of the kernel itself - what a kernel trace reports - and nothing is put into the stream
// between one kernel and the next.  (Events recorded between the kernels instead make the stream drain and write its
// caches back at every kernel boundary; the headline call then read 20 - 30 us longer than it is.)
#pragma once
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include <tuple>
#include <utility>

namespace ccd {

// the stage being timed: `start` goes to the first kernel launched in it, `stop` to every kernel (the last one counts)
struct StageTimer {
  hipEvent_t start, stop;
  bool first;
};
// null unless a timed stage is open (set and cleared by the profiler of infinipot_api.hip, on the calling thread)
extern StageTimer* g_stage_timer;

template <class Tuple, size_t... I>
inline void arg_pointers(Tuple& t, void** out, std::index_sequence<I...>) {
  ((out[I] = (void*)&std::get<I>(t)), ...);
}

template <class... KArgs, class... Args>
inline void launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t s, Args&&... args) {
  static_assert(sizeof...(KArgs) == sizeof...(Args), "argument count of the kernel");
  StageTimer* t = g_stage_timer;
  if (t == nullptr) {
    hipLaunchKernelGGL(kernel, grid, block, 0, s, std::forward<Args>(args)...);
    return;
  }
  std::tuple<KArgs...> formal{std::forward<Args>(args)...};    // converted to the kernel's own parameter types
  void* ptrs[sizeof...(KArgs) ? sizeof...(KArgs) : 1];
  arg_pointers(formal, ptrs, std::index_sequence_for<KArgs...>{});
  (void)hipExtLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, 0, s, t->first ? t->start : nullptr,
                           t->stop, 0);
  t->first = false;
}

}  // namespace ccd
