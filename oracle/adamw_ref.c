/*
 * Scalar reference for the mixed-precision AdamW update of one optimizer-state
 * subgroup.  TEST INFRASTRUCTURE ONLY: it is the slow, one-element-at-a-time
 * definition that the tests, the smoke check and the benchmark's CPU-baseline
 * leg compare the HIP library against.  It shares no code with that library
 * and the library never calls it.
 *
 * What is computed.  The paper (Sections 1, 2 "mixed precision", 4.1) keeps a
 * subgroup's parameters p, momentum m and variance v in FP32, takes 16-bit
 * gradients, updates with Adam (Kingma & Ba) and hands a 16-bit copy of the
 * new parameters back to the model; it prints no update equations.  This file
 * therefore writes out the textbook bias-corrected Adam with decoupled weight
 * decay (AdamW), t being the 1-based index of the step being taken:
 *
 *     m_t = b1*m + (1-b1)*g            v_t = b2*v + (1-b2)*g*g
 *     p_t = p*(1 - lr*wd) - (lr/(1-b1^t)) * m_t / (sqrt(v_t)/sqrt(1-b2^t) + eps)
 *     p_lp = bf16(p_t)                  (round to nearest, ties to even)
 *
 * Precision.  The paper fixes FP32 for the optimizer state, so every
 * per-element operation below is one IEEE-754 binary32 operation, rounded to
 * nearest-even, never fused (build with -ffp-contract=off, no fast-math) and
 * with gradual underflow.  The per-step scalars are formed once in double and
 * rounded to binary32 once.
 *
 * Pins (tests/test_oracle_pins.py): sign-step closed form at t=1, pure decay
 * for zero gradients, geometric recurrences for constant gradients, an
 * independent double-precision evaluation of the textbook formulas, torch's
 * AdamW, element independence by brute force, and an exhaustive check of the
 * bf16 helpers.
 *
 * The end of the file holds the two other adaptive optimizers that Section 4.1
 * names as equally parallel, Adagrad and RMSProp, in the same mixed-precision
 * setting (FP32 p and one FP32 accumulator v, 16-bit gradients in, 16-bit
 * parameters out); their definitions and pins are stated there.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* bf16 is the upper half of a binary32: widening is exact. */
float ref_bf16_to_f32(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return f;
}

/* binary32 -> bf16, round to nearest, ties to even.  NaN stays NaN (made
 * quiet, sign kept); values past the largest finite bf16 round to infinity. */
uint16_t ref_f32_to_bf16(float f) {
  uint32_t u;
  memcpy(&u, &f, sizeof u);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
  uint32_t keep = u >> 16;          /* truncated result            */
  uint32_t rest = u & 0xFFFFu;      /* discarded 16 bits           */
  if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u))) keep += 1u;
  return (uint16_t)keep;
}

/* Array forms of the two helpers (bit patterns in, bit patterns out). */
void ref_bf16_to_f32_n(const uint16_t* in, float* out, uint64_t n) {
  for (uint64_t i = 0; i < n; ++i) out[i] = ref_bf16_to_f32(in[i]);
}
void ref_f32_to_bf16_n(const float* in, uint16_t* out, uint64_t n) {
  for (uint64_t i = 0; i < n; ++i) out[i] = ref_f32_to_bf16(in[i]);
}

typedef struct {
  float beta1, beta2, omb1, omb2, step_size, inv_sqrt_bc2, eps, decay;
} ref_scalars;

/* Per-step scalars: formed in double from the binary32 hyper-parameters, each
 * rounded to binary32 exactly once. */
static ref_scalars ref_make_scalars(float lr, float beta1, float beta2, float eps,
                                    float weight_decay, int64_t step) {
  ref_scalars s;
  double bc1 = 1.0 - pow((double)beta1, (double)step);
  double bc2 = 1.0 - pow((double)beta2, (double)step);
  s.beta1 = beta1;
  s.beta2 = beta2;
  s.omb1 = 1.0f - beta1;
  s.omb2 = 1.0f - beta2;
  s.step_size = (float)((double)lr / bc1);
  s.inv_sqrt_bc2 = (float)(1.0 / sqrt(bc2));
  s.eps = eps;
  s.decay = (float)(1.0 - (double)lr * (double)weight_decay);
  return s;
}

void ref_adamw_scalars(float lr, float beta1, float beta2, float eps, float weight_decay,
                       int64_t step, float out[8]) {
  ref_scalars s = ref_make_scalars(lr, beta1, beta2, eps, weight_decay, step);
  out[0] = s.beta1; out[1] = s.beta2; out[2] = s.omb1; out[3] = s.omb2;
  out[4] = s.step_size; out[5] = s.inv_sqrt_bc2; out[6] = s.eps; out[7] = s.decay;
}

/* One element.  Each statement is one rounded binary32 operation. */
static inline void ref_adamw_element(const ref_scalars* s, float* p, float* m, float* v,
                                     uint16_t g16, uint16_t* p_lp) {
  float g = ref_bf16_to_f32(g16);
  float a = s->beta1 * *m;
  float b = s->omb1 * g;
  float mt = a + b;
  float c = s->beta2 * *v;
  float e = s->omb2 * g;
  float f = e * g;
  float vt = c + f;
  float r = sqrtf(vt);
  float q = r * s->inv_sqrt_bc2;
  float d = q + s->eps;
  float pd = *p * s->decay;          /* decoupled decay acts on the old p */
  float u = mt / d;
  float w = s->step_size * u;
  float pt = pd - w;
  *m = mt;
  *v = vt;
  *p = pt;
  *p_lp = ref_f32_to_bf16(pt);
}

/* Update n elements in place; returns 0, or -1 for arguments the update is not
 * defined for (step < 1, betas outside [0,1), negative eps). */
int ref_adamw_step(float* p, float* m, float* v, const uint16_t* g, uint16_t* p_lp, uint64_t n,
                   float lr, float beta1, float beta2, float eps, float weight_decay,
                   int64_t step) {
  if (step < 1 || !(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f) ||
      !(eps >= 0.0f))
    return -1;
  ref_scalars s = ref_make_scalars(lr, beta1, beta2, eps, weight_decay, step);
  for (uint64_t i = 0; i < n; ++i) ref_adamw_element(&s, &p[i], &m[i], &v[i], g[i], &p_lp[i]);
  return 0;
}

/* The same loop body under a static parallel-for: elements are independent, so
 * the result is bit-identical.  Returns the number of threads used (>= 1), or
 * -1 on invalid arguments. */
int ref_adamw_step_parallel(float* p, float* m, float* v, const uint16_t* g, uint16_t* p_lp,
                            uint64_t n, float lr, float beta1, float beta2, float eps,
                            float weight_decay, int64_t step, int threads) {
  if (step < 1 || !(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f) ||
      !(eps >= 0.0f))
    return -1;
  ref_scalars s = ref_make_scalars(lr, beta1, beta2, eps, weight_decay, step);
  int used = 1;
#ifdef _OPENMP
  if (threads < 1) threads = omp_get_max_threads();
#pragma omp parallel num_threads(threads)
  {
#pragma omp single
    used = omp_get_num_threads();
#pragma omp for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i)
      ref_adamw_element(&s, &p[i], &m[i], &v[i], g[i], &p_lp[i]);
  }
#else
  (void)threads;
  for (uint64_t i = 0; i < n; ++i) ref_adamw_element(&s, &p[i], &m[i], &v[i], g[i], &p_lp[i]);
#endif
  return used;
}

/* ---------------------------------------------------------------------------
 * Adagrad and RMSProp.  Section 4.1 of the paper lists them next to Adam as
 * adaptive optimizers whose update is independent per element; it gives no
 * equations, so these are the textbook rules, with the same decoupled weight
 * decay, eps placement (outside the root) and 16-bit copy as the AdamW above.
 * The state is p and one accumulator v; there is no first moment and no bias
 * correction, so the step index does not enter.
 *
 *   Adagrad (Duchi, Hazan, Singer), diagonal form:
 *       v_t = v + g*g
 *       p_t = p*(1 - lr*wd) - lr * g / (sqrt(v_t) + eps)
 *   RMSProp (the uncentred, momentum-free form):
 *       v_t = alpha*v + (1-alpha)*g*g
 *       p_t = p*(1 - lr*wd) - lr * g / (sqrt(v_t) + eps)
 *
 * Pins (tests/test_oracle_pins.py): first step from v = 0 (sign step, scaled by
 * 1/sqrt(1-alpha) for RMSProp), constant gradients (v_T = T g^2 and the
 * harmonic-root sum for Adagrad; v_t = g^2 (1-alpha^t) for RMSProp), pure decay
 * for zero gradients, an independent double-precision evaluation, torch's
 * Adagrad and RMSprop, element independence.
 */
static inline void ref_accum_tail(float lr, float eps, float decay, float g, float vt, float* p,
                                  float* v, uint16_t* p_lp) {
  float r = sqrtf(vt);
  float d = r + eps;
  float pd = *p * decay;             /* decoupled decay acts on the old p */
  float u = g / d;
  float w = lr * u;
  float pt = pd - w;
  *v = vt;
  *p = pt;
  *p_lp = ref_f32_to_bf16(pt);
}

static inline void ref_adagrad_element(float lr, float eps, float decay, float* p, float* v,
                                       uint16_t g16, uint16_t* p_lp) {
  float g = ref_bf16_to_f32(g16);
  float f = g * g;
  float vt = *v + f;
  ref_accum_tail(lr, eps, decay, g, vt, p, v, p_lp);
}

static inline void ref_rmsprop_element(float lr, float alpha, float oma, float eps, float decay,
                                       float* p, float* v, uint16_t g16, uint16_t* p_lp) {
  float g = ref_bf16_to_f32(g16);
  float c = alpha * *v;
  float e = oma * g;
  float f = e * g;
  float vt = c + f;
  ref_accum_tail(lr, eps, decay, g, vt, p, v, p_lp);
}

/* Update n elements in place.  threads == 1: the plain scalar loop; otherwise
 * the same body under a static parallel-for (threads < 1: all cores).  Returns
 * the number of threads used, or -1 for arguments the update is not defined for
 * (negative eps). */
int ref_adagrad_step(float* p, float* v, const uint16_t* g, uint16_t* p_lp, uint64_t n, float lr,
                     float eps, float weight_decay, int threads) {
  if (!(eps >= 0.0f)) return -1;
  const float decay = (float)(1.0 - (double)lr * (double)weight_decay);
  int used = 1;
  if (threads == 1) {
    for (uint64_t i = 0; i < n; ++i) ref_adagrad_element(lr, eps, decay, &p[i], &v[i], g[i], &p_lp[i]);
    return 1;
  }
#ifdef _OPENMP
  if (threads < 1) threads = omp_get_max_threads();
#pragma omp parallel num_threads(threads)
  {
#pragma omp single
    used = omp_get_num_threads();
#pragma omp for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i)
      ref_adagrad_element(lr, eps, decay, &p[i], &v[i], g[i], &p_lp[i]);
  }
#else
  for (uint64_t i = 0; i < n; ++i) ref_adagrad_element(lr, eps, decay, &p[i], &v[i], g[i], &p_lp[i]);
#endif
  return used;
}

/* As above; also -1 for alpha outside [0, 1). */
int ref_rmsprop_step(float* p, float* v, const uint16_t* g, uint16_t* p_lp, uint64_t n, float lr,
                     float alpha, float eps, float weight_decay, int threads) {
  if (!(eps >= 0.0f) || !(alpha >= 0.0f && alpha < 1.0f)) return -1;
  const float decay = (float)(1.0 - (double)lr * (double)weight_decay);
  const float oma = 1.0f - alpha;
  int used = 1;
  if (threads == 1) {
    for (uint64_t i = 0; i < n; ++i)
      ref_rmsprop_element(lr, alpha, oma, eps, decay, &p[i], &v[i], g[i], &p_lp[i]);
    return 1;
  }
#ifdef _OPENMP
  if (threads < 1) threads = omp_get_max_threads();
#pragma omp parallel num_threads(threads)
  {
#pragma omp single
    used = omp_get_num_threads();
#pragma omp for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i)
      ref_rmsprop_element(lr, alpha, oma, eps, decay, &p[i], &v[i], g[i], &p_lp[i]);
  }
#else
  for (uint64_t i = 0; i < n; ++i)
    ref_rmsprop_element(lr, alpha, oma, eps, decay, &p[i], &v[i], g[i], &p_lp[i]);
#endif
  return used;
}
