// Learnable router: projections, scores and row-wise top-k (Sec. 4, Eq. 16 of the paper; router step of
// Alg. 2), all in fp64 so that the selection agrees with an fp64 reference up to summation order.
//
//   R[i][j] = proj_q(Qbar_i) . proj_k(Kbar_j) / sqrt(d),   proj(x) = x W
//   row i keeps its k largest R[i][j]; equal scores go to the lower j; indices come out ascending.
//
// Two identities keep the work small.  (1) R = (Qbar M) Kbar^T with M = Wq Wk^T / sqrt(d), a d x d
// matrix formed once per call (fold_router_weights, run by spare workgroups of the pooling launch):
// only the 16 query rows of a workgroup are projected, the pooled keys are used as they are.  (2) Kbar is pooled from
// K - colmean(K), which shifts every score of a row by the same amount, (Qbar Wq Wk^T) . colmean(K):
// a row-wise top-k does not see it, so the raw block sums of K are scored and the mean never enters.
// The scores formed here therefore differ from R by one constant per row.
//
// One workgroup of 16 waves handles 16 query blocks of one head.  Scores are formed on the matrix cores
// (v_mfma_f64_16x16x4) 256 key blocks at a time: wave w multiplies the projected 16 x d tile with key
// blocks [256 r + 16 w, +16), parks its 16 x 16 result in LDS, and wave i then picks up row i, so that
// after the last round every wave holds one complete score row in registers (4 values per lane and
// round).  The selection is a most-significant-bit-first search for the k-th largest key on
// order-preserving 64-bit integer images of the scores: counting is a compare plus a scalar popcount
// of the lane mask, there is no sorting and no atomics, and the result does not depend on timing.
// Scores never touch HBM.
#include "common.h"

namespace sla2 {

constexpr int kRouterRows = 16;                       // query blocks per workgroup = waves per workgroup
constexpr int kColsPerRound = 256;                    // key blocks scored per round (16 waves x 16)
constexpr int kStageK = 32;                           // contraction indices per staged operand chunk
constexpr int kStageLd = kStageK + 2;                 // padded row of a staged chunk (doubles)
template <int D> constexpr size_t router_lds_bytes() {
  return sizeof(double) * (kRouterRows * (D + 2) + kRouterRows * (kColsPerRound + 8) + 16 * 16 * kStageLd);
}

// monotone map double -> uint64: a < b  <=>  key(a) < key(b); every real score maps above 0
__device__ __forceinline__ uint64_t order_key(double x) {
  uint64_t u = __builtin_bit_cast(uint64_t, x);
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}

__device__ __forceinline__ int wave_count(bool pred) { return __builtin_popcountll(__ballot(pred)); }

// C[16][D] = A[16][D] M on the matrix cores, M fp64 [D][D] row-major in global memory.  All 16 waves
// work: wave w forms columns [16 (w % (D/16)), +16) over a 1/(16 / (D/16)) share of the contraction
// range; the shares are written side by side (C has room for kShares copies) and added by the reader.
template <int D> struct ProjGeom {
  static constexpr int kNt = D / 16;                 // column tiles
  static constexpr int kShares = 16 / kNt;           // waves per column tile: 2 (D = 128) or 4 (D = 64)
  static constexpr int kSteps = D / 4 / kShares;     // 4-wide contraction steps per wave
};
template <int D>
__device__ __forceinline__ void project16_fetch(double (&b)[ProjGeom<D>::kSteps], const double* __restrict__ M, int wave,
                                                int lane) {
  typedef ProjGeom<D> G;
  const int n = 16 * (wave % G::kNt) + lane % 16, share = wave / G::kNt;
#pragma unroll
  for (int i = 0; i < G::kSteps; i++) b[i] = M[(size_t)(4 * (share * G::kSteps + i) + lane / 16) * D + n];
}
template <int D>
__device__ __forceinline__ void project16(const double (*A)[D + 2], double (*C)[D + 2] /* [kShares*16][D+2] */,
                                          const double (&b)[ProjGeom<D>::kSteps], int wave, int lane) {
  typedef ProjGeom<D> G;
  const int nt = wave % G::kNt, share = wave / G::kNt;
  const int n = 16 * nt + lane % 16;
  f64x4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
  for (int i = 0; i < G::kSteps; i++)
    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(A[lane % 16][4 * (share * G::kSteps + i) + lane / 16], b[i], acc, 0, 0, 0);
#pragma unroll
  for (int v = 0; v < 4; v++) C[share * 16 + lane / 16 + 4 * v][n] = acc[v];
}

template <int D, int SLOTS>
__global__ __launch_bounds__(1024) void router_topk_kernel(const double* __restrict__ q_sum,
                                                           const double* __restrict__ k_sum,
                                                           const double* __restrict__ router_m,
                                                           int32_t* __restrict__ block_idx,
                                                           double* __restrict__ k_mean, int H, int N, int bq, int bk,
                                                           int Tm, int Tn, int k, int w_per_head, int topk_blocks,
                                                           int smooth) {
  // LDS: xa [16][D+2] pooled queries, later Qbar M | tile [16][264] one round of scores (the partial
  // projections before the first round) | stage [16 waves][16][34] each wave's private operand chunk
  extern __shared__ __attribute__((aligned(16))) double lds[];
  double (*xa)[D + 2] = reinterpret_cast<double (*)[D + 2]>(lds);
  double (*tile)[kColsPerRound + 8] = reinterpret_cast<double (*)[kColsPerRound + 8]>(lds + kRouterRows * (D + 2));
  double (*stage)[kStageLd] = reinterpret_cast<double (*)[kStageLd]>(lds + kRouterRows * (D + 2) +
                                                                       kRouterRows * (kColsPerRound + 8)) +
                              (threadIdx.x / kWave) * 16;
  static_assert(ProjGeom<D>::kShares * (D + 2) <= kColsPerRound + 8, "projection shares must fit the score tile");
  double (*xb)[D + 2] = reinterpret_cast<double (*)[D + 2]>(&tile[0][0]);   // partial Qbar M; dead before the first round
  if ((int)blockIdx.x >= topk_blocks) {
    // Spare workgroups of this launch form colmean(K) (K-smoothing step of Alg. 2) from the block sums
    // for the kernels that follow; the router itself does not need it.  16 channels per workgroup,
    // 64 row groups, fixed summation order.  With smoothing disabled the mean is written as zero.
    double* red = &tile[0][0];
    const int job = blockIdx.x - topk_blocks, bh = job / (D / 16), c = 16 * (job % (D / 16)) + threadIdx.x % 16;
    const int g = threadIdx.x / 16;
    double s = 0.0;
    if (smooth)
      for (int j = g; j < Tn; j += 64) s += k_sum[((size_t)bh * Tn + j) * D + c];
    red[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x < 16) {
      double tot = 0.0;
      for (int gi = 0; gi < 64; gi++) tot += red[gi * 16 + threadIdx.x];
      k_mean[(size_t)bh * D + c] = tot / (double)N;
    }
    return;
  }
  const int row_tiles = (Tm + kRouterRows - 1) / kRouterRows;
  const int bh = blockIdx.x / row_tiles;
  const int row0 = (blockIdx.x % row_tiles) * kRouterRows;
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const double* M = router_m + (w_per_head ? (size_t)(bh % H) * D * D : 0);

  double mb[ProjGeom<D>::kSteps];
  project16_fetch<D>(mb, M, wave, lane);               // operands of the projection, in flight during the Qbar load
  for (int e = threadIdx.x; e < kRouterRows * D; e += 1024) {
    const int r = e / D, c = e % D;
    const int row = min(row0 + r, Tm - 1);             // rows past the end repeat the last one; never stored
    const int rows = min(bq, N - row * bq);
    xa[r][c] = q_sum[((size_t)bh * Tm + row) * D + c] / (double)rows;     // mean pooling (Eq. 15)
  }
  __syncthreads();
  project16<D>(xa, xb, mb, wave, lane);                                   // Qbar (Wq Wk^T / sqrt(d)), in shares
  __syncthreads();
  for (int e = threadIdx.x; e < kRouterRows * D; e += 1024) {
    const int r = e / D, c = e % D;
    double v = xb[r][c];
#pragma unroll
    for (int sh = 1; sh < ProjGeom<D>::kShares; sh++) v += xb[sh * 16 + r][c];
    xa[r][c] = v;
  }
  __syncthreads();

  uint64_t key[SLOTS];
#pragma unroll
  for (int s = 0; s < SLOTS; s++) key[s] = 0;

  const int rounds = (Tn + kColsPerRound - 1) / kColsPerRound;
  const double* ks = k_sum + (size_t)bh * Tn * D;
  const double last_cnt = (double)(N - (Tn - 1) * bk);
#pragma unroll
  for (int r = 0; r < SLOTS / 4; r++) {
    if (r < rounds) {
      // --- scores of 16 rows x 16 key blocks on this wave ---
      const int col0 = r * kColsPerRound + wave * 16;
      f64x4 acc = {0.0, 0.0, 0.0, 0.0};
      if (col0 < Tn) {
        // The wave's 16 key rows are fetched with coalesced 16-byte loads (a row's 32 doubles of one
        // chunk are 256 contiguous bytes), one chunk ahead, parked in the wave's private LDS slab and
        // read back in the operand layout of v_mfma_f64_16x16x4 (lane l feeds A[l%16][l/16] and
        // B[l/16][l%16]).  A wave's LDS operations execute in order, so no barrier is involved.
        typedef __attribute__((ext_vector_type(2))) double f64x2;
        const double* kb = ks + (size_t)col0 * D + 2 * (lane % 16);
        f64x2 pre[4];
        auto fetch = [&](int kc) {
#pragma unroll
          for (int i = 0; i < 4; i++) {
            const int r = min(col0 + 4 * i + lane / 16, Tn - 1) - col0;       // rows past the end repeat the last one
            pre[i] = *reinterpret_cast<const f64x2*>(kb + (size_t)r * D + kStageK * kc);
          }
        };
        fetch(0);
#pragma unroll
        for (int kc = 0; kc < D / kStageK; kc++) {
#pragma unroll
          for (int i = 0; i < 4; i++) *reinterpret_cast<f64x2*>(&stage[4 * i + lane / 16][2 * (lane % 16)]) = pre[i];
          if (kc + 1 < D / kStageK) fetch(kc + 1);
#pragma unroll
          for (int kk = 0; kk < kStageK / 4; kk++)
            acc = __builtin_amdgcn_mfma_f64_16x16x4f64(xa[lane % 16][kStageK * kc + 4 * kk + lane / 16],
                                                       stage[lane % 16][4 * kk + lane / 16], acc, 0, 0, 0);
        }
      }
      // result layout: lane l, register v holds C[l/16 + 4 v][l%16]
#pragma unroll
      for (int v = 0; v < 4; v++) tile[lane / 16 + 4 * v][wave * 16 + lane % 16] = acc[v];
      __syncthreads();
      // --- wave i collects row i; block sums -> block means (only a ragged last block differs) ---
#pragma unroll
      for (int qd = 0; qd < 4; qd++) {
        const int col = r * kColsPerRound + qd * kWave + lane;
        double sc = tile[wave][qd * kWave + lane] / (col == Tn - 1 ? last_cnt : (double)bk);
        sc += 0.0;                                     // -0 -> +0: zeros tie
        key[4 * r + qd] = col < Tn ? order_key(sc) : 0ull;
      }
      __syncthreads();
    }
  }

  const int row = row0 + wave;
  if (row >= Tm || k <= 0) return;
  const int slots = rounds * 4;
  int32_t* out = block_idx + ((size_t)bh * Tm + row) * k;

  // k-th largest key thr, most significant bit first, on 32-bit halves (32-bit compares run at full
  // rate).  Invariant of either search: at least `need` candidates are >= the current threshold.
  // `exact` is set as soon as {key >= thr} has exactly k members - no ties to resolve then.
  uint32_t hi[SLOTS], lo[SLOTS];
#pragma unroll
  for (int s = 0; s < SLOTS; s++) { hi[s] = (uint32_t)(key[s] >> 32); lo[s] = (uint32_t)key[s]; }
  uint32_t thr_hi = 0;
  bool exact = false;
  for (int bit = 31; bit >= 0; bit--) {
    const uint32_t cand = thr_hi | (1u << bit);
    int cnt = 0;
#pragma unroll
    for (int s = 0; s < SLOTS; s++) cnt += wave_count(hi[s] >= cand);      // unused slots hold 0 < cand
    if (cnt >= k) {
      thr_hi = cand;
      if (cnt == k) { exact = true; break; }
    }
  }
  uint32_t thr_lo = 0;
  if (!exact) {
    // thr_hi is the high word of the k-th largest key; the keys above it in the high word are in,
    // `need` more come from those that share it, ranked by their low words
    int gt = 0, eq = 0;
#pragma unroll
    for (int s = 0; s < SLOTS; s++) { gt += wave_count(hi[s] > thr_hi); eq += wave_count(hi[s] == thr_hi); }
    const int need = k - gt;
    if (eq == need) {
      exact = true;                                    // all of them: {key >= (thr_hi, 0)} is the answer
    } else {
      for (int bit = 31; bit >= 0; bit--) {
        const uint32_t cand = thr_lo | (1u << bit);
        int cnt = 0;
#pragma unroll
        for (int s = 0; s < SLOTS; s++) cnt += wave_count(hi[s] == thr_hi && lo[s] >= cand);
        if (cnt >= need) {
          thr_lo = cand;
          if (cnt == need) { exact = true; break; }
        }
      }
    }
  }
  const uint64_t thr = ((uint64_t)thr_hi << 32) | thr_lo;
  // not exact: thr is the k-th largest key itself and several keys equal it; those above it
  // are all kept, the equal ones are kept in ascending column order until k are taken.
  int need_eq = 0;
  if (!exact) {
    int gt = 0;
#pragma unroll
    for (int s = 0; s < SLOTS; s++) gt += wave_count(key[s] > thr);
    need_eq = k - gt;
  }
  const uint64_t lane_lt = (1ull << lane) - 1ull;
  int written = 0;
#pragma unroll
  for (int s = 0; s < SLOTS; s++) {
    if (s < slots) {
      bool keep;
      if (exact) {
        keep = key[s] >= thr;
      } else {
        const bool eq = key[s] == thr;
        const uint64_t eq_mask = __ballot(eq);
        const int my_rank = __builtin_popcountll(eq_mask & lane_lt);
        keep = key[s] > thr || (eq && my_rank < need_eq);
        const int taken = __builtin_popcountll(eq_mask);
        need_eq -= taken < need_eq ? taken : need_eq;
      }
      const uint64_t m = __ballot(keep);
      if (keep) out[written + __builtin_popcountll(m & lane_lt)] = s * kWave + lane;
      written += __builtin_popcountll(m);
    }
  }
}

hipError_t launch_router_topk(const Shape& s, const double* q_sum, const double* k_sum, const double* router_m,
                              int32_t* block_idx, double* k_mean, hipStream_t stream) {
  const int row_tiles = (s.Tm + kRouterRows - 1) / kRouterRows;
  const int topk_blocks = s.k > 0 ? s.BH * row_tiles : 0;        // k = 0: only the colmean workgroups run
  dim3 grid((unsigned)(topk_blocks + s.BH * (s.d / 16)));
  const int rounds = (s.Tn + kColsPerRound - 1) / kColsPerRound;     // <= 8 (kMaxKeyBlocks)
#define SLA2_TOPK(DD, SS)                                                                                        \
  {                                                                                                              \
    static OncePerDevice once;                                                                                   \
    if (hipError_t e = allow_dynamic_lds(once, (const void*)router_topk_kernel<DD, SS>, (int)router_lds_bytes<DD>()); \
        e != hipSuccess)                                                                                         \
      return e;                                                                                                  \
    router_topk_kernel<DD, SS><<<grid, 1024, router_lds_bytes<DD>(), stream>>>(                                  \
        q_sum, k_sum, router_m, block_idx, k_mean, s.H, s.N, s.bq, s.bk, s.Tm, s.Tn, s.k, s.w_per_head ? 1 : 0,   \
        topk_blocks, s.smooth ? 1 : 0);                                                                          \
  }
  if (s.d == 128) {
    if (rounds <= 2) SLA2_TOPK(128, 8) else if (rounds <= 4) SLA2_TOPK(128, 16) else SLA2_TOPK(128, 32)
  } else {
    if (rounds <= 2) SLA2_TOPK(64, 8) else if (rounds <= 4) SLA2_TOPK(64, 16) else SLA2_TOPK(64, 32)
  }
#undef SLA2_TOPK
  return hipGetLastError();
}

}  // namespace sla2
