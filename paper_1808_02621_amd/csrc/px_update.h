// The two optimizer updates, element-wise, shared by the stand-alone apply kernel and by the
// fused aggregate-and-apply path so that both produce the same bits.
//   gradient descent:  w <- w - lr * g
//   Adagrad:           a <- a + g * g ;  w <- w - lr * g / (sqrt(a) + eps)      (updated a)
#ifndef PX_UPDATE_H_
#define PX_UPDATE_H_

#include <hip/hip_runtime.h>

namespace pxu {

__device__ __forceinline__ void sgd(float& w, float g, float lr) { w = fmaf(-lr, g, w); }

__device__ __forceinline__ void adagrad(float& w, float& a, float g, float lr, float eps) {
    a = fmaf(g, g, a);
    w = w - (lr * g) / (sqrtf(a) + eps);
}

}  // namespace pxu

#endif  // PX_UPDATE_H_
