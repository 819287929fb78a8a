// The per-element parameter update, shared by the streaming optimizer kernel and the fused
// weight-gradient epilogue so that both produce the same bits (paper, Approach, "Desiderata": the
// update must be exactly the one unsharded training applies, whichever kernel applies it).
//   SGD:  p <- p - lr g
//   Adam: m <- b1 m + c1 g;  v <- b2 v + c2 g^2;  p <- p - lr (m bc1) / (sqrt(v bc2) + eps)
// with c = 1 - b and bc = 1/(1 - b^t) rounded from double by the host.
// Every operation is a single correctly rounded fp32 operation in a fixed order: contraction is
// switched off here, so the compiler cannot fuse differently in different callers.
#pragma once
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace hydra {

template <int OPT>
__device__ __forceinline__ void optim_step(float& p, float& m, float& v, const float g, const OptimHp& h) {
#pragma clang fp contract(off)
  if (OPT == 0) {
    const float d = h.lr * g;
    p = p - d;
  } else {
    const float t1 = h.b1 * m, u1 = h.c1 * g;
    m = t1 + u1;
    const float t2 = h.b2 * v, u2 = h.c2 * g;
    const float u3 = u2 * g;
    v = t2 + u3;
    const float mh = m * h.bc1, vh = v * h.bc2;
    const float den = __builtin_sqrtf(vh) + h.eps;
    const float q = h.lr * mh;
    const float d = q / den;
    p = p - d;
  }
}

}  // namespace hydra
