// SoftTop-k router (Sec. 6 of the paper): the differentiable stand-in for the hard block selection that
// the first training stage uses,
//      M[i][j] = sigmoid(P_c[i][j] / tau + lambda_i),   P_c = row softmax of the router scores,
// with lambda_i found by bisection so that row i sums to k.  One workgroup per query block i; fp64
// throughout (the row sum decides lambda_i).  Inputs are the pooled sums and the folded router matrix
// that the pooling kernel leaves in the workspace.  This is a training-time operator: it is written
// to be plainly correct and deterministic (fixed reduction order), not tuned.
#include "common.h"

namespace sla2 {

__device__ __forceinline__ double sigmoid_f64(double x) {
  const double e = exp(-fabs(x));
  return x >= 0.0 ? 1.0 / (1.0 + e) : e / (1.0 + e);
}

// sum of v over the 256 threads, same order on every call; result on all threads
__device__ __forceinline__ double block_sum(double v, double* red /* LDS [256] */) {
  __syncthreads();
  red[threadIdx.x] = v;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  return red[0];
}
__device__ __forceinline__ double block_max(double v, double* red) {
  __syncthreads();
  red[threadIdx.x] = v;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] = fmax(red[threadIdx.x], red[threadIdx.x + s]);
    __syncthreads();
  }
  return red[0];
}

__global__ __launch_bounds__(256) void router_soft_kernel(const double* __restrict__ q_sum,
                                                          const double* __restrict__ k_sum,
                                                          const double* __restrict__ router_m,
                                                          float* __restrict__ mask, int H, int N, int d, int bq,
                                                          int bk, int Tm, int Tn, int k, double tau,
                                                          int w_per_head) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  double* x = reinterpret_cast<double*>(smem_raw);        // [Tn]: scores, then P_c / tau
  double* y = x + Tn;                                     // [d]: pooled query row times the folded matrix
  double* qb = y + d;                                     // [d]: pooled query row
  double* red = qb + d;                                   // [256]
  const int bh = blockIdx.x / Tm, i = blockIdx.x % Tm, h = bh % H, tid = threadIdx.x;
  float* out = mask + ((size_t)bh * Tm + i) * Tn;
  if (k <= 0 || k >= Tn) {                                // the limits lambda -> -inf / +inf
    for (int j = tid; j < Tn; j += 256) out[j] = k <= 0 ? 0.f : 1.f;
    return;
  }
  const double* M = router_m + (w_per_head ? (size_t)h * d * d : 0);
  const double q_cnt = (double)min(bq, N - i * bq);
  if (tid < d) qb[tid] = q_sum[((size_t)bh * Tm + i) * d + tid] / q_cnt;
  __syncthreads();
  if (tid < d) {                                          // y = qbar M  (M = Wq Wk^T / sqrt d, Eq. 16)
    double acc = 0.0;
    for (int a = 0; a < d; a++) acc += qb[a] * M[(size_t)a * d + tid];
    y[tid] = acc;
  }
  __syncthreads();
  // scores against the pooled keys.  The smoothing shift of K moves a whole row of scores by one
  // constant, which the row softmax cancels: the raw block sums are used.
  double mx = -INFINITY;
  for (int j = tid; j < Tn; j += 256) {
    const double* kr = k_sum + ((size_t)bh * Tn + j) * d;
    double acc = 0.0;
    for (int c = 0; c < d; c++) acc += y[c] * kr[c];
    acc /= (double)min(bk, N - j * bk);
    x[j] = acc;
    mx = fmax(mx, acc);
  }
  mx = block_max(mx, red);
  double se = 0.0;
  for (int j = tid; j < Tn; j += 256) {
    const double e = exp(x[j] - mx);
    x[j] = e;
    se += e;
  }
  se = block_sum(se, red);
  double xmin = INFINITY, xmax = -INFINITY;
  for (int j = tid; j < Tn; j += 256) {
    const double v = x[j] / se / tau;
    x[j] = v;
    xmin = fmin(xmin, v);
    xmax = fmax(xmax, v);
  }
  xmax = block_max(xmax, red);
  xmin = -block_max(-xmin, red);
  // bisection on a bracket that contains the root (the row sum is increasing in lambda): every
  // thread follows the same lo / hi, so the loop is uniform; it ends when the interval stops shrinking
  const double logit = log((double)k / (double)(Tn - k));
  double lo = logit - xmax - 1e-9, hi = logit - xmin + 1e-9;
  for (int it = 0; it < 200; it++) {
    const double mid = 0.5 * (lo + hi);
    if (mid <= lo || mid >= hi) break;
    double s = 0.0;
    for (int j = tid; j < Tn; j += 256) s += sigmoid_f64(x[j] + mid);
    s = block_sum(s, red);
    if (s < (double)k) lo = mid;
    else hi = mid;
  }
  const double lam = 0.5 * (lo + hi);
  for (int j = tid; j < Tn; j += 256) out[j] = (float)sigmoid_f64(x[j] + lam);
}

hipError_t launch_router_soft(const Shape& s, const double* q_sum, const double* k_sum, const double* router_m,
                              float* mask, double tau, hipStream_t stream) {
  const size_t smem = ((size_t)s.Tn + 2 * s.d + 256) * sizeof(double);
  router_soft_kernel<<<dim3((unsigned)(s.BH * s.Tm)), 256, smem, stream>>>(q_sum, k_sum, router_m, mask, s.H, s.N,
                                                                           s.d, s.bq, s.bk, s.Tm, s.Tn, s.k, tau,
                                                                           s.w_per_head ? 1 : 0);
  return hipGetLastError();
}

}  // namespace sla2
