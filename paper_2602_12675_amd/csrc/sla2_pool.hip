// Pooling side of the learnable router (Sec. 4, Eq. 15 of the paper; pooling step of Alg. 2): sums of
// the rows of every query block and key block, accumulated in fp64 so that the block selection
// downstream agrees with an fp64 reference up to summation order.
//
// This is a bandwidth kernel: it streams Q and K once with 16-byte loads and is bound by HBM.
#include <type_traits>

#include "common.h"

namespace sla2 {

template <typename T> struct Vec16;
template <> struct Vec16<uint16_t> {
  static constexpr int kElems = 8;
  typedef u32x4 Raw;
  __device__ static Raw load_raw(const uint16_t* p) { return *reinterpret_cast<const u32x4*>(p); }
  __device__ static void unpack(Raw u, float (&f)[8]) {
#pragma unroll
    for (int i = 0; i < 4; i++) {
      f[2 * i] = __builtin_bit_cast(float, u[i] << 16);
      f[2 * i + 1] = __builtin_bit_cast(float, u[i] & 0xFFFF0000u);
    }
  }
};
template <> struct Vec16<float> {
  static constexpr int kElems = 4;
  typedef f32x4 Raw;
  __device__ static Raw load_raw(const float* p) { return *reinterpret_cast<const f32x4*>(p); }
  __device__ static void unpack(Raw u, float (&f)[4]) { f[0] = u[0]; f[1] = u[1]; f[2] = u[2]; f[3] = u[3]; }
};

// Row `a` of M = Wq Wk^T / sqrt(d):  M[a][c] = sum_n Wq[a][n] Wk[c][n] / sqrt(d)   (Eq. 16, both router
// projections folded into one d x d matrix), fp64 throughout.  256 threads: thread (c, part) sums a
// 1/(256/d) share of n for column c, with all of its loads in flight at once; shares meet in LDS.
__device__ void fold_router_row(const float* __restrict__ Wq, const float* __restrict__ Wk, double* __restrict__ M,
                                int d, int a, double* red /* LDS [256] */) {
  const int c = threadIdx.x % d, part = threadIdx.x / d, parts = 256 / d;
  const int n0 = part * (d / parts);
  constexpr int kBatch = 4;                            // loads in flight per operand; the pooling path sets the register budget
  f32x4 wk[kBatch], wq[kBatch];                        // d / parts / 4 = 16 (d = 128) or 4 (d = 64) groups of 4
  double acc = 0.0;
  for (int h = 0; h < d / parts / 4; h += kBatch) {
#pragma unroll
    for (int x = 0; x < kBatch; x++) {
      const int n = n0 + 4 * (h + x);
      const bool ok = h + x < d / parts / 4;
      wk[x] = ok ? *reinterpret_cast<const f32x4*>(Wk + (size_t)c * d + n) : f32x4{0.f, 0.f, 0.f, 0.f};
      wq[x] = ok ? *reinterpret_cast<const f32x4*>(Wq + (size_t)a * d + n) : f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int x = 0; x < kBatch; x++)
#pragma unroll
      for (int e = 0; e < 4; e++) acc += (double)wq[x][e] * (double)wk[x][e];
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  if (threadIdx.x < d) {
    double tot = 0.0;
    for (int pi = 0; pi < parts; pi++) tot += red[pi * d + threadIdx.x];
    M[(size_t)a * d + c] = tot / sqrt((double)d);
  }
}

// One workgroup (256 threads) per block of Q or of K; each thread owns EPL consecutive channels of
// one row per pass and has all of its 16-byte loads in flight at once; partial sums meet in LDS in a
// fixed order.  Thousands of small workgroups keep enough bytes in flight to stream at HBM speed.
template <typename T>
__global__ __launch_bounds__(256) void block_sums_kernel(const T* __restrict__ q, const T* __restrict__ k,
                                                         double* __restrict__ q_sum, double* __restrict__ k_sum,
                                                         Strides sin, int H, int N, int d, int bq, int bk, int Tm,
                                                         int Tn, int fold_blocks,
                                                         const float* __restrict__ router_w,
                                                         double* __restrict__ router_m) {
  constexpr int EPL = Vec16<T>::kElems;
  __shared__ double red[2048];               // [row group][channel]: at most 32 groups x 64 ch or 16 x 128
  if ((int)blockIdx.x < fold_blocks) {
    // the first workgroups of this launch fold the router weights, one row of M each, for every weight
    // pair; they finish long before the pooling workgroups behind them
    const int pair = blockIdx.x / d, a = blockIdx.x % d;
    const float* Wq = router_w + (size_t)pair * 2 * d * d;
    fold_router_row(Wq, Wq + (size_t)d * d, router_m + (size_t)pair * d * d, d, a, red);
    return;
  }
  const int pool_id = blockIdx.x - fold_blocks;
  const int per_head = Tm + Tn;
  const int bh = pool_id / per_head;
  int t = pool_id % per_head;
  const bool is_k = t >= Tm;
  if (is_k) t -= Tm;
  const int b = is_k ? bk : bq;
  const T* x = (is_k ? k : q) + head_offset(sin, bh, H);
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
  const T* px = x + (size_t)(row0 + rg) * sin.n + col;
  const size_t pass_stride = (size_t)rpp * sin.n;
  // A full block is a known number of passes: every load of the thread is issued before the first
  // sum (a loop with a run-time trip count leaves one load in flight at a time and a round trip
  // to memory per pass).
  auto full = [&](auto loads_tag) {
    constexpr int LOADS = decltype(loads_tag)::value;
    typename Vec16<T>::Raw raw[LOADS];
#pragma unroll
    for (int i = 0; i < LOADS; i++) raw[i] = Vec16<T>::load_raw(px + i * pass_stride);
#pragma unroll
    for (int i = 0; i < LOADS; i++) {      // ascending rows, as the run-time loop below
      float f[EPL];
      Vec16<T>::unpack(raw[i], f);
#pragma unroll
      for (int e = 0; e < EPL; e++) acc[e] += (double)f[e];
    }
  };
  // passes per full block: b / rpp = 2, 4 or 8 for bf16 rows, 4, 8 or 16 for fp32 rows
  const int passes = (rows == b && b % rpp == 0) ? b / rpp : 0;
  if (passes == 4) full(std::integral_constant<int, 4>());
  else if (passes == 8) full(std::integral_constant<int, 8>());
  else if (passes == 2 && EPL == 8) full(std::integral_constant<int, 2>());
  else if (passes == 16 && EPL == 4) full(std::integral_constant<int, EPL == 4 ? 16 : 2>());
  else {
#pragma unroll 4
    for (int r = rg; r < rows; r += rpp) {
      float f[EPL];
      Vec16<T>::unpack(Vec16<T>::load_raw(x + (size_t)(row0 + r) * sin.n + col), f);
#pragma unroll
      for (int e = 0; e < EPL; e++) acc[e] += (double)f[e];
    }
  }
#pragma unroll
  for (int e = 0; e < EPL; e++) red[rg * d + col + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < d) {
    double s = 0.0;
    for (int gi = 0; gi < rpp; gi++) s += red[gi * d + threadIdx.x];
    out[threadIdx.x] = s;
  }
}

hipError_t launch_block_sums(const Shape& s, const void* q, const void* k, const float* router_w, double* q_sum,
                             double* k_sum, double* router_m, hipStream_t stream) {
  const int fold_blocks = (s.w_per_head ? s.H : 1) * s.d;
  dim3 grid((unsigned)(s.BH * (s.Tm + s.Tn) + fold_blocks));
  if (s.bf16)
    block_sums_kernel<uint16_t><<<grid, 256, 0, stream>>>((const uint16_t*)q, (const uint16_t*)k, q_sum, k_sum, s.sin,
                                                           s.H, s.N, s.d, s.bq, s.bk, s.Tm, s.Tn, fold_blocks, router_w,
                                                           router_m);
  else
    block_sums_kernel<float><<<grid, 256, 0, stream>>>((const float*)q, (const float*)k, q_sum, k_sum, s.sin, s.H, s.N,
                                                        s.d, s.bq, s.bk, s.Tm, s.Tn, fold_blocks, router_w, router_m);
  return hipGetLastError();
}

}  // namespace sla2
