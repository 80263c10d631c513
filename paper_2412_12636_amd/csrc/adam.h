// The Adam update of one element, shared by the flat sweep and by the weight-gradient product whose epilogue
// applies it.  Contraction is switched off inside, so that both places round every operation the same way and
// give the same bits.
#pragma once
#include <math.h>

#include "common.h"

namespace tmk {

struct AdamScalars {
  float lr, beta1, beta2, one_minus_beta1, one_minus_beta2, eps, weight_decay, grad_scale, inv_bc1, inv_bc2;
};

__device__ __forceinline__ void adam_one(float &p, float g, float &m, float &v, const AdamScalars &a) {
#pragma clang fp contract(off)
  g *= a.grad_scale;
  m = a.beta1 * m + a.one_minus_beta1 * g;
  v = a.beta2 * v + a.one_minus_beta2 * g * g;
  const float mhat = m * a.inv_bc1;
  const float vhat = v * a.inv_bc2;
  p = p - a.lr * (mhat / (sqrtf(vhat) + a.eps) + a.weight_decay * p);
}

// bias-correction scalars and differences are formed in double on the host: 1 - 0.999 in fp32 is off by 6e-5
inline AdamScalars make_adam_scalars(const tm_adam_hparams_t *hp, int64_t step) {
  AdamScalars a;
  a.lr = (float)hp->lr;
  a.beta1 = (float)hp->beta1;
  a.beta2 = (float)hp->beta2;
  a.one_minus_beta1 = (float)(1.0 - hp->beta1);
  a.one_minus_beta2 = (float)(1.0 - hp->beta2);
  a.eps = (float)hp->eps;
  a.weight_decay = (float)hp->weight_decay;
  a.grad_scale = (float)hp->grad_scale;
  a.inv_bc1 = (float)(1.0 / (1.0 - pow(hp->beta1, (double)step)));
  a.inv_bc2 = (float)(1.0 / (1.0 - pow(hp->beta2, (double)step)));
  return a;
}

// State of the parameters a weight-gradient product covers, for the product's fused update: element (n, k) of
// the gradient belongs to master[n*ldc + k] and so on.
struct AdamTarget {
  float *master, *exp_avg, *exp_avg_sq;
  bf16 *lowp;  // bf16 copy of the parameters
  int store_grad;  // 0: the gradient is consumed in registers and never stored
  AdamScalars a;
};

// Up to eight stretches of one flat state for one launch of the update: element ranges and the first block of each.
constexpr int kAdamMaxSegments = 8;
struct AdamSegments {
  int n;
  int block0[kAdamMaxSegments];
  int64_t first[kAdamMaxSegments], count[kAdamMaxSegments];
};

}  // namespace tmk
