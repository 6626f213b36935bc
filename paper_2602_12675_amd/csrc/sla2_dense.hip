// Dense attention softmax(Q K^T / sqrt(d)) V in bf16 for d = 128: the comparator the SLA2 speed-ups are
// quoted against (Sec. 9.1 of the paper: C = 4 N^2 d).
//
// One workgroup = 8 waves = 256 query rows, one workgroup per CU, two waves per SIMD.  A tile of 64 keys is
// two phases for a wave: a vector phase (online softmax of its 32 x 64 scores) and a matrix phase (O^T += V^T P^T of
// this tile, then S^T = K Q^T of the next one).  A SIMD runs vector and matrix instructions side by side
// only if they come from different waves, so the two waves of a SIMD are kept in opposite phases: waves
// 4-7 run half a tile behind waves 0-3, and every phase ends in a workgroup barrier.  While one wave of a
// SIMD feeds the matrix pipe the other one has the vector unit to itself.
//
// K and V tiles go global -> LDS (swizzled layout, see mfma_tiles.h) through three buffers: tile t is read from
// half-step 2t - 1 (its K, by the leading waves) to 2t + 2 (its V, by the trailing ones); tile t + 2 is requested in
// half-step 2t + 2, into the buffer tile t - 1 has just left, and has landed by the end of half-step 2t + 3.
// All LDS operand reads are issued by hand and waited for by count (they are consumed within the phase that
// issued them); the softmax keeps its reference while the row maximum stays within 2^8 of it.
#include "mfma_tiles.h"

namespace sla2 {

template <int D> struct DenseSmem {
  static constexpr int kTile = SwizzledLayout<D>::kTileBytes;              // one 64 x D bf16 tile
  static constexpr int kBuf = 2 * kTile;                                   // K then V
  static constexpr int kLoop = 3 * kBuf;
  static constexpr int kLd = D + 8;
  static constexpr int kEpi = 256 * kLd * 2;                               // output tile [256][D + 8]
  static constexpr int kBytes = kLoop > kEpi ? kLoop : kEpi;
};

// lanes l and l ^ 32 combine their values through v_permlane32_swap (a vector instruction: no LDS round trip,
// whose latency a wave that has the vector unit to itself would sit out)
__device__ __forceinline__ float swap_halves_max(float x) {
  const unsigned u = __builtin_bit_cast(unsigned, x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);   // r[0] = low half twice, r[1] = high half twice
  return fmaxf(__builtin_bit_cast(float, (unsigned)r[0]), __builtin_bit_cast(float, (unsigned)r[1]));
}
__device__ __forceinline__ float swap_halves_sum(float x) {
  const unsigned u = __builtin_bit_cast(unsigned, x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __builtin_bit_cast(float, (unsigned)r[0]) + __builtin_bit_cast(float, (unsigned)r[1]);
}
// Between two phases.  LDS is written by the tile transfers only (waited for through vmcnt where a phase
// needs them), and every operand read is waited for by the product that consumes it, so the barrier itself
// waits for nothing: reads issued before it stay in flight across it.
__device__ __forceinline__ void phase_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

template <int D>
__global__ __launch_bounds__(512, 1) void dense_pp_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                          const uint16_t* __restrict__ v, uint16_t* __restrict__ out,
                                                          Strides sin, Strides sout, int H, int N, int Tm, int Tn) {
  constexpr int BQ = 256, NW = 8, KS = D / 16, ET = D / 32, LD = D + 8;
  typedef DenseSmem<D> SM;
  typedef SwizzledLayoutB<D> SL;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const int per_head = (Tm + kXcds - 1) / kXcds;
  const int bh = (blockIdx.x / kXcds) / per_head, i = (blockIdx.x % kXcds) * per_head + (blockIdx.x / kXcds) % per_head;
  if (i >= Tm) return;
  const int tid = threadIdx.x, lane = tid % kWave, g = lane / 32;
  const int w = __builtin_amdgcn_readfirstlane(tid / kWave);
  const bool trailing = w >= 4;                       // waves 4-7 run half a tile behind waves 0-3
  const int row0 = i * BQ;
  const int rows_valid = min(BQ, N - row0);
  const int qrow = 32 * w + lane % 32;
  const uint16_t* qh = q + head_offset(sin, bh, H);
  const uint16_t* kh = k + head_offset(sin, bh, H);
  const uint16_t* vh = v + head_offset(sin, bh, H);
  const int tok_stride = sin.n;
  const int n = Tn;
  auto kbuf = [&](int t) { return reinterpret_cast<uint16_t*>(smem + (t % 3) * SM::kBuf); };
  auto vbuf = [&](int t) { return reinterpret_cast<uint16_t*>(smem + (t % 3) * SM::kBuf + SM::kTile); };
  // tile t: K and V, 2 + 2 transfers of 1 KB per wave (rows past the end repeat the last one: their scores are masked)
  auto dma = [&](int t) {
    const int t0 = t * kTileTokens, valid = min(kTileTokens, N - t0);
    dma_tile<D, NW, SL>(kh + (size_t)t0 * tok_stride, tok_stride, valid, kbuf(t), w, lane);
    dma_tile<D, NW, SL>(vh + (size_t)t0 * tok_stride, tok_stride, valid, vbuf(t), w, lane);
  };
  dma(0);
  if (n > 1) dma(1);
  // Q fragments (B operand of S^T = K Q^T): lane <- Q[row][16 ks + 8 g + 0..7]
  bf16x8 qf[KS];
  {
    const int r = min(qrow, rows_valid - 1);
    const uint16_t* src = qh + (size_t)(row0 + r) * tok_stride + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) qf[ks] = *reinterpret_cast<const bf16x8*>(src + 16 * ks);
  }
  __builtin_amdgcn_s_waitcnt(kVmcnt0);
  phase_barrier();                                    // tiles 0 and 1 are in LDS for everyone

  f32x16 oacc[ET], sacc[2];
#pragma unroll
  for (int et = 0; et < ET; et++)
#pragma unroll
    for (int e = 0; e < 16; e++) oacc[et][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;               // reference of the exponentials and running sum, log2 domain
  const float c1 = kLog2e * rsqrtf((float)D);
  bf16x8 pf[4];

  // S^T = K_t Q^T (keys x query rows), two 32-key halves.  The operand of (ks, mt) is 16 bytes of key row
  // 32 mt + l % 32; in the swizzled tile it sits at (address of ks = 0) ^ 32 ks.  Reads run two steps ahead.
  auto scores = [&](int t) {
    const unsigned ka = lds_address(kbuf(t)) + (unsigned)(lane % 32) * (D * 2) + 16u * (unsigned)(g ^ SL::swz(lane % 16));
    constexpr int KA = 2;                             // steps of the head dimension the reads run ahead of the products
    u32x4 kr[KA + 1][2];
#pragma unroll
    for (int ks = 0; ks < KA; ks++) {
      kr[ks][0] = lds_read16_untracked<0>(ka ^ (32u * ks));
      kr[ks][1] = lds_read16_untracked<32 * D * 2>(ka ^ (32u * ks));
    }
#pragma unroll
    for (int mt = 0; mt < 2; mt++)
#pragma unroll
      for (int e = 0; e < 16; e++) sacc[mt][e] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      if (ks + KA < KS) {
        kr[(ks + KA) % (KA + 1)][0] = lds_read16_untracked<0>(ka ^ (32u * (ks + KA)));
        kr[(ks + KA) % (KA + 1)][1] = lds_read16_untracked<32 * D * 2>(ka ^ (32u * (ks + KA)));
      }
      const int ahead = KS - 1 - ks < KA ? KS - 1 - ks : KA;
#pragma unroll
      for (int mt = 0; mt < 2; mt++) {
        wait_lgkmcnt(2 * ahead + 1 - mt);
        settle(kr[ks % (KA + 1)][mt]);
        sacc[mt] = mfma_bf16(__builtin_bit_cast(bf16x8, kr[ks % (KA + 1)][mt]), qf[ks], sacc[mt]);
      }
    }
  };
  // online softmax of this lane's query row over the 64 keys of tile t: P^T fragments in token order, rescaling of O^T
  auto softmax = [&](int t) {
    const int valid = min(kTileTokens, N - t * kTileTokens);
    if (valid < kTileTokens) {
#pragma unroll
      for (int mt = 0; mt < 2; mt++)
#pragma unroll
        for (int e = 0; e < 16; e++)
          if (32 * mt + 8 * (e / 4) + 4 * g + e % 4 >= valid) sacc[mt][e] = -INFINITY;
    }
    float mx = -INFINITY;
#pragma unroll
    for (int mt = 0; mt < 2; mt++)
#pragma unroll
      for (int e = 0; e < 16; e++) mx = fmaxf(mx, sacc[mt][e]);
    mx = swap_halves_max(mx) * c1;
    // the reference is kept while the row maximum stays within 2^8 of it (decided for the whole wave)
    const bool rescale = __builtin_amdgcn_ballot_w64(mx > m_run + 8.f) != 0;
    const float m_new = rescale ? fmaxf(m_run, mx) : m_run;
    float rs = 0.f;
#pragma unroll
    for (int mt = 0; mt < 2; mt++)
#pragma unroll
      for (int e = 0; e < 16; e += 2) {
        const float p0 = fast_exp2(sacc[mt][e] * c1 - m_new);
        const float p1 = fast_exp2(sacc[mt][e + 1] * c1 - m_new);
        rs += p0 + p1;
        pf[2 * mt + e / 8][e % 8] = (__bf16)p0;
        pf[2 * mt + e / 8][e % 8 + 1] = (__bf16)p1;
      }
    rs = swap_halves_sum(rs);
    if (rescale) {
      const float corr = fast_exp2(m_run - m_new);    // 0 on the first tile
      l_run *= corr;
      m_run = m_new;
#pragma unroll
      for (int et = 0; et < ET; et++)
#pragma unroll
        for (int e = 0; e < 16; e++) oacc[et][e] *= corr;
    }
    l_run += rs;
  };
  // O^T += V_t^T P^T: fragment (ks, et) = two transposing reads, kept three fragments ahead of the products
  constexpr int kAhead = 3, kFrags = (kTileTokens / 16) * ET;
  u32x2 vlo[kAhead + 1], vhi[kAhead + 1];
  unsigned va_lo = 0, va_hi = 0;
  // the first reads of the values phase, issued at the end of the softmax phase: their latency passes while the
  // wave waits at the barrier between the two
  auto values_prefetch = [&](int t) {
    const uint16_t* vt = vbuf(t);
    // fragment (ks, et): rows 16 ks + 4 g + 0..3 ("lo") and 16 ks + 8 + 4 g + 0..3 ("hi"); the position of a chunk
    // depends on row % 16 only, so the token step is an immediate and the channel tile an XOR on the address
    const int vcol = 16 * ((lane / 16) % 2) + 4 * (lane % 4);
    va_lo = lds_address(vt + SL::offset(4 * g + (lane % 16) / 4, vcol));
    va_hi = lds_address(vt + SL::offset(8 + 4 * g + (lane % 16) / 4, vcol));
#pragma unroll
    for (int f = 0; f < kAhead; f++) {
      vlo[f] = lds_read_tr_untracked_at<16 * D * 2>(va_lo ^ (64u * (f % ET)), f / ET);
      vhi[f] = lds_read_tr_untracked_at<16 * D * 2>(va_hi ^ (64u * (f % ET)), f / ET);
    }
  };
  auto values = [&]() {
#pragma unroll
    for (int f = 0; f < kFrags; f++) {
      if (f + kAhead < kFrags) {
        const int f2 = f + kAhead;
        vlo[f2 % (kAhead + 1)] = lds_read_tr_untracked_at<16 * D * 2>(va_lo ^ (64u * (f2 % ET)), f2 / ET);
        vhi[f2 % (kAhead + 1)] = lds_read_tr_untracked_at<16 * D * 2>(va_hi ^ (64u * (f2 % ET)), f2 / ET);
      }
      const int left = kFrags - 1 - f;
      wait_lgkmcnt(2 * (left < kAhead ? left : kAhead));
      u32x2& lo = vlo[f % (kAhead + 1)];
      u32x2& hi = vhi[f % (kAhead + 1)];
      settle(lo);
      settle(hi);
      const u32x4 v4 = {lo[0], lo[1], hi[0], hi[1]};
      oacc[f % ET] = mfma_bf16(__builtin_bit_cast(bf16x8, v4), pf[f / ET], oacc[f % ET]);
    }
  };

  // Half-steps h = 0 .. 2 n + 1, a barrier after each.  Leading waves: h = 0 scores of tile 0; h = 2 s + 1 softmax of
  // tile s; h = 2 s + 2 values of tile s and scores of tile s + 1.  Trailing waves: the same, one half-step later.
  // Tile t + 2 is requested in half-step 2 t + 2 (tile t - 1 was last read in half-step 2 t + 1) and must have
  // landed by the end of half-step 2 t + 3: every odd half-step ends with a wait for this wave's transfers.
  // For a leading wave the odd half-steps are the softmax phases, for a trailing wave the values phases.
  if (trailing) phase_barrier();                      // half-step 0: the leading waves form their first scores
  scores(0);
  phase_barrier();
  for (int s = 0; s < n; s++) {
    // ---- vector phase ----
    if (trailing && s + 2 < n) dma(s + 2);            // half-step 2 s + 2
    softmax(s);
    values_prefetch(s);
    if (!trailing) __builtin_amdgcn_s_waitcnt(kVmcnt0);   // half-step 2 s + 1
    phase_barrier();
    // ---- matrix phase ----
    if (!trailing && s + 2 < n) dma(s + 2);           // half-step 2 s + 2
    values();
    if (s + 1 < n) scores(s + 1);
    if (trailing) __builtin_amdgcn_s_waitcnt(kVmcnt0);    // half-step 2 s + 3
    phase_barrier();
  }
  if (!trailing) phase_barrier();                     // half-step 2 n + 1: the trailing waves finish
  __builtin_amdgcn_s_waitcnt(kVmcnt0);

  // ---- normalise, transpose through LDS, coalesced store ----
  uint16_t* os = reinterpret_cast<uint16_t*>(smem);
  const float inv_l = l_run > 0.f ? 1.f / l_run : 0.f;
#pragma unroll
  for (int et = 0; et < ET; et++)
#pragma unroll
    for (int v4 = 0; v4 < 4; v4++) {
      bf16x4 pk;
#pragma unroll
      for (int r = 0; r < 4; r++) pk[r] = (__bf16)(inv_l * oacc[et][4 * v4 + r]);
      *reinterpret_cast<bf16x4*>(os + qrow * LD + 32 * et + 8 * v4 + 4 * g) = pk;
    }
  __syncthreads();
  uint16_t* oh = out + head_offset(sout, bh, H) + (size_t)row0 * sout.n;
  for (int idx = tid; idx < BQ * (D / 8); idx += NW * kWave) {
    const int r = idx / (D / 8), ch = idx % (D / 8);
    if (r < rows_valid) *reinterpret_cast<u32x4*>(oh + (size_t)r * sout.n + 8 * ch) = *reinterpret_cast<const u32x4*>(os + r * LD + 8 * ch);
  }
}

hipError_t launch_dense_pp(const Shape& s, const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* out,
                           hipStream_t stream) {
  constexpr int smem = DenseSmem<128>::kBytes;
  static OncePerDevice once;
  if (hipError_t e = allow_dynamic_lds(once, (const void*)dense_pp_kernel<128>, smem); e != hipSuccess) return e;
  const int Tm = (s.N + 255) / 256;
  const int grid = ((Tm + kXcds - 1) / kXcds) * kXcds * s.BH;
  dense_pp_kernel<128><<<dim3((unsigned)grid), 512, smem, stream>>>(q, k, v, out, s.sin, s.sout, s.H, s.N, Tm, s.Tn);
  return hipGetLastError();
}

}  // namespace sla2
