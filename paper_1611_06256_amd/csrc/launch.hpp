// One place through which every kernel of the library is launched.
//
// Normally a plain launch.  While a stage timer is open on the calling host thread (the optional per-stage timing of
// the library), the launch carries an event pair of its own: the runtime stamps those two events with the start and
// the end of that very dispatch, so the elapsed time between them is the kernel's execution time, the figure a
// kernel trace shows, without the queueing and dispatch latency that two events recorded around a launch include.
#pragma once
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include <tuple>
#include <utility>

namespace ga3c {

struct LaunchTimer {
    // hands out the events of the next launch; false = launch untimed
    virtual bool next_events(hipEvent_t *start, hipEvent_t *stop) = 0;

protected:
    ~LaunchTimer() = default;
};

// the open stage timer of this host thread, if any
inline thread_local LaunchTimer *launch_timer = nullptr;

namespace detail {
template <typename... KArgs, size_t... I>
inline hipError_t launch_timed(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t s, hipEvent_t a,
                               hipEvent_t b, std::tuple<KArgs...> &args, std::index_sequence<I...>) {
    void *ptrs[sizeof...(KArgs) > 0 ? sizeof...(KArgs) : 1] = {(void *)&std::get<I>(args)...};
    return hipExtLaunchKernel((const void *)kernel, grid, block, ptrs, lds, s, a, b, 0);
}
}  // namespace detail

// kernel<<<grid, block, lds, s>>>(args...); the arguments convert to the kernel's parameter types as in a call.
template <typename... KArgs, typename... Args>
inline void launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t s, Args &&...args) {
    static_assert(sizeof...(KArgs) == sizeof...(Args), "one argument per kernel parameter");
    hipEvent_t a = nullptr, b = nullptr;
    if (launch_timer && launch_timer->next_events(&a, &b)) {
        std::tuple<KArgs...> held{static_cast<KArgs>(args)...};
        (void)detail::launch_timed(kernel, grid, block, lds, s, a, b, held, std::index_sequence_for<KArgs...>{});
        return;
    }
    hipLaunchKernelGGL(kernel, grid, block, lds, s, static_cast<KArgs>(args)...);
}

}  // namespace ga3c
