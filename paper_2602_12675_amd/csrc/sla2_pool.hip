// Pooling side of the learnable router (Sec. 4, Eq. 15-16 of the paper; pooling
// and K-smoothing steps of Alg. 2): block sums of Q and K, colmean(K), and the
// two d x d projections.  Everything is accumulated in fp64 so that the block
// selection downstream agrees with an fp64 reference up to summation order.
//
// block_sums is the bandwidth kernel of the three: it streams Q and K once
// (16-byte loads, one workgroup per block) and is bound by HBM.
#include "common.h"

namespace sla2 {

// ---------------------------------------------------------------------------------------------
// block sums: out[bh][t][c] = sum over the rows of block t of x[bh][row][c]
// One workgroup (256 threads) per block of Q or of K; each thread owns EPL consecutive
// channels of one row per pass, partial sums meet in LDS in a fixed order.
// ---------------------------------------------------------------------------------------------
template <typename T> struct Vec16;
template <> struct Vec16<uint16_t> {
  static constexpr int kElems = 8;
  __device__ static void load(const uint16_t* p, float (&f)[8]) {
    uint4 u = *reinterpret_cast<const uint4*>(p);
    uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; i++) {
      f[2 * i] = __builtin_bit_cast(float, w[i] << 16);
      f[2 * i + 1] = __builtin_bit_cast(float, w[i] & 0xFFFF0000u);
    }
  }
};
template <> struct Vec16<float> {
  static constexpr int kElems = 4;
  __device__ static void load(const float* p, float (&f)[4]) {
    float4 u = *reinterpret_cast<const float4*>(p);
    f[0] = u.x; f[1] = u.y; f[2] = u.z; f[3] = u.w;
  }
};

template <typename T>
__global__ __launch_bounds__(256) void block_sums_kernel(const T* __restrict__ q, const T* __restrict__ k,
                                                         double* __restrict__ q_sum, double* __restrict__ k_sum,
                                                         int N, int d, int bq, int bk, int Tm, int Tn) {
  constexpr int EPL = Vec16<T>::kElems;
  __shared__ double red[2048];               // [row group][channel]: at most 32 groups x 64 ch or 16 x 128
  const int per_head = Tm + Tn;
  const int bh = blockIdx.x / per_head;
  int t = blockIdx.x % per_head;
  const bool is_k = t >= Tm;
  if (is_k) t -= Tm;
  const int b = is_k ? bk : bq;
  const T* x = (is_k ? k : q) + (size_t)bh * N * d;
  double* out = (is_k ? k_sum + ((size_t)bh * Tn + t) * d : q_sum + ((size_t)bh * Tm + t) * d);

  const int tpr = d / EPL;                   // threads per row
  const int rpp = 256 / tpr;                 // rows per pass
  const int col = (threadIdx.x % tpr) * EPL;
  const int rg = threadIdx.x / tpr;          // row group
  const int row0 = t * b;
  const int rows = min(b, N - row0);

  double acc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; e++) acc[e] = 0.0;
#pragma unroll 4
  for (int r = rg; r < rows; r += rpp) {
    float f[EPL];
    Vec16<T>::load(x + (size_t)(row0 + r) * d + col, f);
#pragma unroll
    for (int e = 0; e < EPL; e++) acc[e] += (double)f[e];
  }
#pragma unroll
  for (int e = 0; e < EPL; e++) red[rg * d + col + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < d) {
    double s = 0.0;
    for (int g = 0; g < rpp; g++) s += red[g * d + threadIdx.x];
    out[threadIdx.x] = s;
  }
}

hipError_t launch_block_sums(const Shape& s, const void* q, const void* k, double* q_sum, double* k_sum,
                             hipStream_t stream) {
  dim3 grid((unsigned)(s.BH * (s.Tm + s.Tn)));
  if (s.bf16)
    block_sums_kernel<uint16_t><<<grid, 256, 0, stream>>>((const uint16_t*)q, (const uint16_t*)k, q_sum, k_sum, s.N,
                                                           s.d, s.bq, s.bk, s.Tm, s.Tn);
  else
    block_sums_kernel<float><<<grid, 256, 0, stream>>>((const float*)q, (const float*)k, q_sum, k_sum, s.N, s.d, s.bq,
                                                        s.bk, s.Tm, s.Tn);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// colmean(K) = (sum over blocks of the block sums) / N          (K-smoothing step of Alg. 2)
// One workgroup per head.  With smoothing disabled the mean is written as zero so that
// every consumer can subtract it unconditionally.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void col_mean_kernel(const double* __restrict__ k_sum, double* __restrict__ k_mean,
                                                        int N, int d, int Tn, int smooth) {
  __shared__ double red[1024];
  const int bh = blockIdx.x;
  const int c = threadIdx.x % d, g = threadIdx.x / d, G = 1024 / d;
  double s = 0.0;
  if (smooth)
    for (int j = g; j < Tn; j += G) s += k_sum[((size_t)bh * Tn + j) * d + c];
  red[threadIdx.x] = s;
  __syncthreads();
  if (threadIdx.x < d) {
    double tot = 0.0;
    for (int gg = 0; gg < G; gg++) tot += red[gg * d + threadIdx.x];
    k_mean[(size_t)bh * d + threadIdx.x] = tot / (double)N;
  }
}

hipError_t launch_col_mean(const Shape& s, const double* k_sum, double* k_mean, hipStream_t stream) {
  col_mean_kernel<<<dim3((unsigned)s.BH), 1024, 0, stream>>>(k_sum, k_mean, s.N, s.d, s.Tn, s.smooth ? 1 : 0);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// projections: q_proj = (q_sum / rows) Wq / sqrt(d),  k_proj = (k_sum / rows - colmean K) Wk    (Eq. 16)
// One workgroup of d threads per 16 pooled rows; thread c owns output channel c.
// W is [d_in, d_out] row-major, so the threads of a wave read consecutive floats of one W row.
// ---------------------------------------------------------------------------------------------
constexpr int kProjRows = 16;

__global__ __launch_bounds__(128) void project_kernel(const double* __restrict__ q_sum, const double* __restrict__ k_sum,
                                                      const double* __restrict__ k_mean,
                                                      const float* __restrict__ router_w, double* __restrict__ q_proj,
                                                      double* __restrict__ k_proj, int N, int d, int bq, int bk, int Tm,
                                                      int Tn, int H, int w_per_head) {
  __shared__ double x[kProjRows][128];
  const int tiles_q = (Tm + kProjRows - 1) / kProjRows, tiles_k = (Tn + kProjRows - 1) / kProjRows;
  const int per_head = tiles_q + tiles_k;
  const int bh = blockIdx.x / per_head;
  int tile = blockIdx.x % per_head;
  const bool is_k = tile >= tiles_q;
  if (is_k) tile -= tiles_q;
  const int T = is_k ? Tn : Tm, b = is_k ? bk : bq;
  const double* src = (is_k ? k_sum : q_sum) + (size_t)bh * T * d;
  double* dst = (is_k ? k_proj : q_proj) + (size_t)bh * T * d;
  const float* W = router_w + (w_per_head ? (size_t)(bh % H) * 2 * d * d : 0) + (is_k ? (size_t)d * d : 0);
  const int c = threadIdx.x;
  const int r0 = tile * kProjRows;
  const double mu = is_k ? k_mean[(size_t)bh * d + c] : 0.0;
  for (int r = 0; r < kProjRows; r++) {
    int row = r0 + r;
    double v = 0.0;
    if (row < T) {
      int rows = min(b, N - row * b);
      v = src[(size_t)row * d + c] / (double)rows - mu;
    }
    x[r][c] = v;
  }
  __syncthreads();
  double acc[kProjRows];
#pragma unroll
  for (int r = 0; r < kProjRows; r++) acc[r] = 0.0;
  for (int e = 0; e < d; e++) {
    double w = (double)W[(size_t)e * d + c];
#pragma unroll
    for (int r = 0; r < kProjRows; r++) acc[r] += x[r][e] * w;
  }
  const double scale = is_k ? 1.0 : 1.0 / sqrt((double)d);
  for (int r = 0; r < kProjRows; r++)
    if (r0 + r < T) dst[(size_t)(r0 + r) * d + c] = acc[r] * scale;
}

hipError_t launch_project(const Shape& s, const double* q_sum, const double* k_sum, const double* k_mean,
                          const float* router_w, double* q_proj, double* k_proj, hipStream_t stream) {
  int tiles = (s.Tm + kProjRows - 1) / kProjRows + (s.Tn + kProjRows - 1) / kProjRows;
  project_kernel<<<dim3((unsigned)(s.BH * tiles)), s.d, 0, stream>>>(q_sum, k_sum, k_mean, router_w, q_proj, k_proj,
                                                                     s.N, s.d, s.bq, s.bk, s.Tm, s.Tn, s.H,
                                                                     s.w_per_head ? 1 : 0);
  return hipGetLastError();
}

}  // namespace sla2
