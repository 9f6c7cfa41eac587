// opt_elem.h -- the per-element arithmetic shared by the update and averaging kernels (gfx950).
#pragma once
#include <hip/hip_runtime.h>

namespace qsr {

// AdamW (decoupled weight decay, bias-corrected), in the order
//   m <- m + (1-b1)(g - m) ; v <- v + (1-b2)(g^2 - v)
//   theta <- theta - [ eta*lambda*theta + (eta/bc1) * m / (sqrt(v)/sqrt(bc2) + eps) ]
// The moment updates are written as one rounding on top of the old moment, and the decay and
// the Adam step are added before they are subtracted from theta, so that each state variable
// takes one rounding per step (keeps thousands of fp32 steps within 1e-5 of exact arithmetic).
__device__ __forceinline__ void adamw_elem(float &th, float g, float &m, float &v, float etalam,
                                           float stepsz, float rsq_bc2, float c1, float c2,
                                           float eps)
{
    m = fmaf(c1, g - m, m);
    v = fmaf(c2, fmaf(g, g, -v), v);
    float denom = fmaf(sqrtf(v), rsq_bc2, eps);
    float upd = (stepsz * m) / denom;
    th = th - fmaf(etalam, th, upd);
}

// SGD with heavy-ball momentum and coupled weight decay:
//   g' = g + lambda*theta ; buf <- mu*buf + g' ; theta <- theta - eta*buf
__device__ __forceinline__ void sgdm_elem(float &th, float g, float &buf, float eta, float mu,
                                          float lambda)
{
    float gp = fmaf(lambda, th, g);
    buf = fmaf(mu, buf, gp);
    th = fmaf(-eta, buf, th);
}

// s + c <- s + c + r, with the rounding error of s + r recovered exactly (two-sum)
__device__ __forceinline__ void add_comp(float &s, float &c, float r)
{
    float t = s + r;
    float bp = t - s;
    c += (s - (t - bp)) + (r - bp);
    s = t;
}

}  // namespace qsr
