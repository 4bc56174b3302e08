/*
 * fp64 CPU oracle of the optimiser step that follows the backward pass.
 *
 * TEST INFRASTRUCTURE ONLY (see lobra_oracle.c): shares nothing with the HIP sources.
 *
 * The paper trains every task's adapter with Adam and cites both Adam and its decoupled
 * weight-decay form (section 5.1, experimental setup).  This is that algorithm as published
 * (Kingma & Ba, Algorithm 1; Loshchilov & Hutter, Algorithm 2), taken step by step, one
 * independent update per parameter element, with per-task learning rate, step count and
 * gradient scale because every task of the fused batch is its own fine-tuning job:
 *
 *     g     = scale_t * grad
 *     m     = beta1 m + (1 - beta1) g
 *     v     = beta2 v + (1 - beta2) g^2
 *     mhat  = m / (1 - beta1^k_t)          k_t = 1-based count of the step being taken
 *     vhat  = v / (1 - beta2^k_t)
 *     theta = theta - lr_t * ( mhat / (sqrt(vhat) + eps) + wd * theta )
 *
 * The parameters of all tasks are stacked by rank row: rows rank_off[t] .. rank_off[t+1]-1 of a
 * [R_tot, d] matrix belong to task t.
 *
 * Pins (tests/test_adam.py): torch.optim.AdamW in fp64 over several steps, the closed form of the
 * first step, the fixed point at zero gradient, invariance to the gradient's scale when eps = 0.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

int lobra_oracle_adam(int32_t n_tasks, const int32_t *rank_off, int32_t d,
                      const double *lr, const int32_t *step, const double *scale,
                      double beta1, double beta2, double eps, double wd,
                      const double *grad, double *theta, double *m, double *v)
{
    for (int32_t t = 0; t < n_tasks; ++t) {
        if (step[t] < 1)
            return -1;
        const double c1 = 1.0 - pow(beta1, (double)step[t]);
        const double c2 = 1.0 - pow(beta2, (double)step[t]);
        for (int32_t R = rank_off[t]; R < rank_off[t + 1]; ++R)
            for (int32_t j = 0; j < d; ++j) {
                const size_t i = (size_t)R * d + j;
                const double g = scale[t] * grad[i];
                m[i] = beta1 * m[i] + (1.0 - beta1) * g;
                v[i] = beta2 * v[i] + (1.0 - beta2) * g * g;
                const double mhat = m[i] / c1;
                const double vhat = v[i] / c2;
                theta[i] = theta[i] - lr[t] * (mhat / (sqrt(vhat) + eps) + wd * theta[i]);
            }
    }
    return 0;
}
