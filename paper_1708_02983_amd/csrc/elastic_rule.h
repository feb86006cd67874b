// The worker rules of the elastic update, shared by the streaming update kernels and by the
// matrix-product epilogue that applies them to a freshly computed gradient tile.
#pragma once
#include <hip/hip_runtime.h>

namespace easgd {

// One worker's rule applied to T = float or a float vector.  Returns d = w - c (time-t values).
template <bool MOM, typename T>
__device__ __forceinline__ T worker_rule(T &w, T &v, T g, T c, float eta, float rho, float alpha, float delta)
{
    const T d = w - c;
    if constexpr (MOM) {
        v = delta * v - eta * g;              // Eq. (5)
        w = (w + v) - alpha * d;              // Eq. (6)
    } else {
        w = w - eta * (g + rho * d);          // Eq. (1)
    }
    return d;
}

}  // namespace easgd
