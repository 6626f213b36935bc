// Router scores and row-wise top-k (Sec. 4, Eq. 16 of the paper; router step of Alg. 2).
//
//   R[i][j] = q_proj[i] . k_proj[j]          (the 1/sqrt(d) is already folded into q_proj)
//   row i keeps its k largest R[i][j]; equal scores go to the lower j; indices come out ascending.
//
// One workgroup of 16 waves handles 16 query blocks of one head.  Scores are formed in fp64 on
// the matrix cores (v_mfma_f64_16x16x4) 256 key blocks at a time: wave w multiplies the 16 x d
// tile of q_proj with key blocks [256 r + 16 w, +16), parks its 16 x 16 result in LDS, and wave i
// then picks up row i, so that after the last round every wave holds one complete score row in
// registers (4 values per lane and round).  The selection is a most-significant-bit-first
// search for the k-th largest key on order-preserving 64-bit integer images of the scores:
// counting is a compare plus a scalar popcount of the lane mask, there is no sorting and no
// atomics, and the result does not depend on timing.  Scores never touch HBM.
#include "common.h"

namespace sla2 {

constexpr int kRouterRows = 16;                       // query blocks per workgroup = waves per workgroup
constexpr int kColsPerRound = 256;                    // key blocks scored per round (16 waves x 16)
constexpr int kMaxSlots = kMaxKeyBlocks / kWave;      // score slots per lane

// monotone map double -> uint64: a < b  <=>  key(a) < key(b); every real score maps above 0
__device__ __forceinline__ uint64_t order_key(double x) {
  uint64_t u = __builtin_bit_cast(uint64_t, x);
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}

__device__ __forceinline__ int wave_count(bool pred) { return __builtin_popcountll(__ballot(pred)); }

template <int D>
__global__ __launch_bounds__(1024) void router_topk_kernel(const double* __restrict__ q_proj,
                                                           const double* __restrict__ k_proj,
                                                           int32_t* __restrict__ block_idx, int Tm, int Tn, int k) {
  __shared__ double qp[kRouterRows][D + 2];            // +2: rows land in different banks
  __shared__ double tile[kRouterRows][kColsPerRound + 2];
  const int row_tiles = (Tm + kRouterRows - 1) / kRouterRows;
  const int bh = blockIdx.x / row_tiles;
  const int row0 = (blockIdx.x % row_tiles) * kRouterRows;
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;

  for (int e = threadIdx.x; e < kRouterRows * D; e += 1024) {
    int r = e / D, c = e % D;
    int row = min(row0 + r, Tm - 1);                   // rows past the end repeat the last one; never stored
    qp[r][c] = q_proj[((size_t)bh * Tm + row) * D + c];
  }
  __syncthreads();

  uint64_t key[kMaxSlots];
#pragma unroll
  for (int s = 0; s < kMaxSlots; s++) key[s] = 0;

  const int rounds = (Tn + kColsPerRound - 1) / kColsPerRound;
  const double* kp = k_proj + (size_t)bh * Tn * D;
#pragma unroll
  for (int r = 0; r < kMaxSlots / 4; r++) {
    if (r < rounds) {
      // --- scores of 16 rows x 16 key blocks on this wave ---
      const int col0 = r * kColsPerRound + wave * 16;
      f64x4 acc = {0.0, 0.0, 0.0, 0.0};
      if (col0 < Tn) {
        // operand layout of v_mfma_f64_16x16x4: lane l feeds A[l%16][l/16] and B[l/16][l%16]
        const int jrow = min(col0 + lane % 16, Tn - 1);
        const double* kb = kp + (size_t)jrow * D + lane / 16;
        const double* qa = &qp[lane % 16][lane / 16];
#pragma unroll 8
        for (int kk = 0; kk < D / 4; kk++)
          acc = __builtin_amdgcn_mfma_f64_16x16x4f64(qa[4 * kk], kb[4 * kk], acc, 0, 0, 0);
      }
      // result layout: lane l, register v holds C[l/16 + 4 v][l%16]
#pragma unroll
      for (int v = 0; v < 4; v++) tile[lane / 16 + 4 * v][wave * 16 + lane % 16] = acc[v];
      __syncthreads();
      // --- wave i collects row i ---
#pragma unroll
      for (int qd = 0; qd < 4; qd++) {
        int col = r * kColsPerRound + qd * kWave + lane;
        double sc = tile[wave][qd * kWave + lane] + 0.0;   // -0 -> +0: zeros tie
        key[4 * r + qd] = col < Tn ? order_key(sc) : 0ull;
      }
      __syncthreads();
    }
  }

  const int row = row0 + wave;
  if (row >= Tm || k <= 0) return;
  const int slots = rounds * 4;
  int32_t* out = block_idx + ((size_t)bh * Tm + row) * k;

  // k-th largest key, most significant bit first.  Invariant: count(key >= thr) >= k.
  uint64_t thr = 0;
  bool exact = false;                                  // true: {key >= thr} has exactly k members
  for (int bit = 63; bit >= 0; bit--) {
    uint64_t cand = thr | (1ull << bit);
    int cnt = 0;
#pragma unroll
    for (int s = 0; s < kMaxSlots; s++)
      if (s < slots) cnt += wave_count(key[s] >= cand);
    if (cnt >= k) {
      thr = cand;
      if (cnt == k) { exact = true; break; }
    }
  }
  // not exact: thr is the k-th largest key itself and several keys equal it; those above it
  // are all kept, the equal ones are kept in ascending column order until k are taken.
  int need_eq = 0;
  if (!exact) {
    int gt = 0;
#pragma unroll
    for (int s = 0; s < kMaxSlots; s++)
      if (s < slots) gt += wave_count(key[s] > thr);
    need_eq = k - gt;
  }
  const uint64_t lane_lt = (1ull << lane) - 1ull;
  int written = 0;
#pragma unroll
  for (int s = 0; s < kMaxSlots; s++) {
    if (s < slots) {
      bool keep;
      if (exact) {
        keep = key[s] >= thr;
      } else {
        bool eq = key[s] == thr;
        uint64_t eq_mask = __ballot(eq);
        int my_rank = __builtin_popcountll(eq_mask & lane_lt);
        keep = key[s] > thr || (eq && my_rank < need_eq);
        int taken = __builtin_popcountll(eq_mask);
        need_eq -= taken < need_eq ? taken : need_eq;
      }
      uint64_t m = __ballot(keep);
      if (keep) out[written + __builtin_popcountll(m & lane_lt)] = s * kWave + lane;
      written += __builtin_popcountll(m);
    }
  }
}

hipError_t launch_router_topk(const Shape& s, const double* q_proj, const double* k_proj, int32_t* block_idx,
                              hipStream_t stream) {
  int row_tiles = (s.Tm + kRouterRows - 1) / kRouterRows;
  dim3 grid((unsigned)(s.BH * row_tiles));
  if (s.d == 128)
    router_topk_kernel<128><<<grid, 1024, 0, stream>>>(q_proj, k_proj, block_idx, s.Tm, s.Tn, s.k);
  else
    router_topk_kernel<64><<<grid, 1024, 0, stream>>>(q_proj, k_proj, block_idx, s.Tm, s.Tn, s.k);
  return hipGetLastError();
}

}  // namespace sla2
