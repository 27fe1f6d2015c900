/* Host build of the device math header (plain C): lets the CPU tests compare the exact
 * functions the kernels use with libm, value by value. */
#include "q8_math.h"

void q8m_tanh(const float *x, float *y, long n) { for (long i = 0; i < n; ++i) y[i] = q8_tanh_rn(x[i]); }
void q8m_sigmoid(const float *x, float *y, long n) { for (long i = 0; i < n; ++i) y[i] = q8_sigmoid_rn(x[i]); }
void q8m_exp(const double *x, double *y, long n) { for (long i = 0; i < n; ++i) y[i] = q8_exp_d(x[i]); }
