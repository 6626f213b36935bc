// Backward pass of SLA2 on the matrix cores, for bf16 tensors (Alg. 3 of the paper's appendix with the
// steps it leaves to automatic differentiation written out; Sec. 5: the backward pass is never
// quantised).  Products run as v_mfma_f32_32x32x16_bf16 with fp32 accumulation; everything between
// them (exp, the D^s / D^l terms, both softmax-backward steps) is fp32.
//
// In each kernel the scores are laid out so that the probabilities feed the next product from registers:
//
//   bwd_q_mfma   one workgroup per query block i (b_q rows, one wave per 32 rows), scores transposed as
//                in the forward kernel, S^T = K Q^T (keys x query rows): one lane owns one query row, so
//                L and D^s are per-lane scalars and dS^T is the B operand of the product that contracts
//                over keys.  Over the selected key blocks: P^T = exp(S^T - L), dP^T = V dO^T,
//                dS^T = P^T (.) (alpha dP^T - D^s), dQ^T += K^T dS^T.  Then the linear branch from the
//                H_i^T, Z_i the forward pass kept: dQ^phi^T = (1 - alpha) H_i dO^T - Z_i D^l^T (over
//                Q^phi Z_i), dQ += softmax-backward(dQ^phi), dH_i = (Q^phi / (Q^phi Z_i))^T dO^l, dZ_i.
//   bwd_kv_mfma  one workgroup per key block j, over the query blocks that selected it, 64 rows a
//                step: here S = Q K^T (rows x keys), so that P and dS are already laid out as the
//                B operands of dV^T += dO^T (alpha P), dK'^T += Q^T dS.  Then the linear branch:
//                dH = dH_total - sum over those query blocks of dH_i (Alg. 3's M_c[i, j] = 0 sum, by
//                complement), dK^phi^T = dH V^T + dZ 1^T, dV^T += dH^T K^phi^T,
//                dK' += softmax-backward(dK^phi).
#include <type_traits>

#include "mfma_tiles.h"

namespace sla2 {

// ---------------------------------------------------------------------------------------------
template <int D, int BQ> struct BwdQSmem {
  static constexpr int kLd = D + 8;
  static constexpr int kTile = SwizzledLayout<D>::kTileBytes;                  // one 64 x D bf16 tile
  static constexpr int kLoopBytes = 4 * kTile;                                 // two buffers of (K, V)
  static constexpr int kEpiA = (D > BQ ? D : BQ) * kLd * 2;                    // H_i^T [D][kLd], the dQ tile, dO [BQ][kLd]
  static constexpr int kEpiB = BQ * kLd * 2;                                   // w [BQ][kLd]
  static constexpr int kTiles = kLoopBytes > kEpiA + kEpiB ? kLoopBytes : kEpiA + kEpiB;
  static constexpr int kZsOff = kTiles;                                        // float [D]   Z_i
  static constexpr int kMuOff = kZsOff + D * 4;                                // float [D]   colmean(K)
  static constexpr int kDlOff = kMuOff + D * 4;                                // float [BQ]  D^l per row
  static constexpr int kRedOff = kDlOff + BQ * 4;                              // float [8]
  static constexpr int kBytes = kRedOff + 32;
};

template <int D, int BQ>
__global__ __launch_bounds__(BQ * 2, 2) void bwd_q_mfma_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const uint16_t* __restrict__ dout, const uint16_t* __restrict__ o_s, const float* __restrict__ lse,
    const double* __restrict__ k_mean, const uint16_t* __restrict__ h_i,
    const float* __restrict__ z_i, const int32_t* __restrict__ block_idx, const float* __restrict__ alpha,
    uint16_t* __restrict__ dq, float* __restrict__ ds_out, float* __restrict__ lraw_out, uint16_t* __restrict__ dh_out,
    float* __restrict__ dz_out, float* __restrict__ dalpha_part, Strides sin, Strides sout, int H, int N, int Tm, int Tn,
    int ksel, int alpha_per_block) {
  constexpr int NW = BQ / 32, NT = NW * kWave;
  constexpr int LD = D + 8, KS = D / 16, ET = D / 32;
  typedef SwizzledLayout<D> SL;
  typedef PaddedLayout<D> PL;
  typedef BwdQSmem<D, BQ> SM;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  float* zs = reinterpret_cast<float*>(smem + SM::kZsOff);
  float* mus = reinterpret_cast<float*>(smem + SM::kMuOff);
  float* dls = reinterpret_cast<float*>(smem + SM::kDlOff);
  float* red = reinterpret_cast<float*>(smem + SM::kRedOff);
  auto kbuf = [&](int buf) { return reinterpret_cast<uint16_t*>(smem + buf * 2 * SM::kTile); };
  auto vbuf = [&](int buf) { return reinterpret_cast<uint16_t*>(smem + buf * 2 * SM::kTile + SM::kTile); };

  // consecutive query blocks of a head share key/value tiles: every head is cut into 8 runs of
  // consecutive blocks, one per XCD (own L2), and all XCDs work through the heads in the same order
  const int per_head = (Tm + kXcds - 1) / kXcds;
  const int bh = (blockIdx.x / kXcds) / per_head, i = (blockIdx.x % kXcds) * per_head + (blockIdx.x / kXcds) % per_head;
  if (i >= Tm) return;
  const int h = bh % H;
  const int tid = threadIdx.x, lane = tid % kWave, g = lane / 32;
  const int w = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int row0 = i * BQ;
  const int rows_valid = min(BQ, N - row0);
  const int qrow = 32 * w + lane % 32;               // this lane's query row inside the block
  const bool row_ok = qrow < rows_valid;
  const int r_ld = min(qrow, rows_valid - 1);        // rows past the end repeat the last one; never stored
  const uint16_t* qh = q + head_offset(sin, bh, H);
  const uint16_t* kh = k + head_offset(sin, bh, H);
  const uint16_t* vh = v + head_offset(sin, bh, H);
  const uint16_t* doh = dout + head_offset(sout, bh, H);
  const int tok_stride = sin.n;
  const int32_t* sel = block_idx + ((size_t)bh * Tm + i) * ksel;
  const int ntiles = ksel;
  const float al = alpha[alpha_per_block ? (size_t)h * Tm + i : (size_t)h];
  const float rscale = rsqrtf((float)D);
  const size_t slot = (size_t)bh * Tm + i;

  auto dma = [&](int j, int buf) {
    const int t0 = j * kTileTokens, valid = min(kTileTokens, N - t0);
    dma_tile<D, NW>(kh + (size_t)t0 * tok_stride, tok_stride, valid, kbuf(buf), w, lane);
    dma_tile<D, NW>(vh + (size_t)t0 * tok_stride, tok_stride, valid, vbuf(buf), w, lane);
  };
  int j_cur = ntiles > 0 ? sel[0] : 0, j_nxt = ntiles > 1 ? sel[1] : 0;
  if (ntiles > 0) dma(j_cur, 0);
  if (tid < D) mus[tid] = (float)k_mean[(size_t)bh * D + tid];

  // ---- prologue: Q and dO as B-operand fragments (alpha is applied to the products); dO . O^s per row ----
  bf16x8 qf[KS], gof[KS];
  float dot_s = 0.f;                                 // dO . O^s of this lane's row;  D^s = alpha dot_s
  {
    const uint16_t* qsrc = qh + (size_t)(row0 + r_ld) * tok_stride + 8 * g;
    const uint16_t* gsrc = doh + (size_t)(row0 + r_ld) * sout.n + 8 * g;
    const uint16_t* ossrc = o_s + ((size_t)bh * N + row0 + r_ld) * D + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      qf[ks] = *reinterpret_cast<const bf16x8*>(qsrc + 16 * ks);
      gof[ks] = *reinterpret_cast<const bf16x8*>(gsrc + 16 * ks);
      const bf16x8 os = *reinterpret_cast<const bf16x8*>(ossrc + 16 * ks);
#pragma unroll
      for (int e = 0; e < 8; e++) dot_s += (float)gof[ks][e] * (float)os[e];
    }
  }
  dot_s = half_sum(dot_s);
  const float Ds = al * dot_s;
  const float L = lse[(size_t)bh * N + row0 + r_ld];
  __builtin_amdgcn_s_waitcnt(kVmcnt0);               // tile 0 and everything above have landed
  __syncthreads();                                   // ... for everyone; mus is visible
  // The forward pass defines L on the smoothed keys; the products below use the raw K, whose scores are
  // larger by q . colmean(K) / sqrt(d) in every column of a row.
  float qmu = 0.f;
#pragma unroll
  for (int ks = 0; ks < KS; ks++) {
    const f32x4 m0 = *reinterpret_cast<const f32x4*>(mus + 16 * ks + 8 * g);
    const f32x4 m1 = *reinterpret_cast<const f32x4*>(mus + 16 * ks + 8 * g + 4);
#pragma unroll
    for (int e = 0; e < 8; e++) qmu += (float)qf[ks][e] * (e < 4 ? m0[e] : m1[e - 4]);
  }
  qmu = half_sum(qmu);
  const float Lraw = L + qmu * rscale;
  const float L2 = Lraw * kLog2e;
  if (g == 0 && row_ok) {
    ds_out[(size_t)bh * N + row0 + qrow] = Ds;
    lraw_out[(size_t)bh * N + row0 + qrow] = L2;      // as the key-side kernel uses it: L on the raw keys, times log2(e)
  }

  // LDS byte offsets of this lane's operand reads inside a K or V tile: row-wise reads (key row
  // l % 32, channel step ks at (offset of step 0) ^ 32 ks) and transposing reads (cf. read_tr4)
  const unsigned b_off = (unsigned)SL::offset(lane % 32, 8 * g) * 2;
  unsigned a_off[ET];
#pragma unroll
  for (int et = 0; et < ET; et++)
    a_off[et] = (unsigned)SL::offset(4 * g + (lane % 16) / 4, 32 * et + 16 * ((lane / 16) % 2) + 4 * (lane % 4)) * 2;
  f32x16 dqacc[ET];
#pragma unroll
  for (int et = 0; et < ET; et++)
#pragma unroll
    for (int e = 0; e < 16; e++) dqacc[et][e] = 0.f;
  float sumds = 0.f;
  const float c0 = kLog2e * rscale;

  for (int s = 0; s < ntiles; s++) {
    const int buf = s & 1;
    const int valid = min(kTileTokens, N - j_cur * kTileTokens);
    const int j_nn = sel[min(s + 2, ntiles - 1)];
    if (s + 1 < ntiles) dma(j_nxt, buf ^ 1);
    j_cur = j_nxt;
    j_nxt = j_nn;
    const unsigned ka = lds_address(kbuf(buf)), va = lds_address(vbuf(buf));
    f32x16 sacc[2], dpacc[2];
#pragma unroll
    for (int mt = 0; mt < 2; mt++)
#pragma unroll
      for (int e = 0; e < 16; e++) { sacc[mt][e] = 0.f; dpacc[mt][e] = 0.f; }
    // S^T = K Q^T and dP^T = V dO^T (keys x query rows; alpha joins below), two 32-key halves each.  One operand read
    // (16 bytes of key row 32 mt + l % 32) per product, issued untracked and kept kAhead deep in flight:
    // a tracked read would be waited for right before its product, one LDS round trip per product.
    {
      constexpr int kItems = 4 * KS, kAhead = 6, kSlots = kAhead + 1;
      u32x4 ring[kSlots];
      auto issue = [&](int n) {                      // item n: (K | V, key half, channel step)
        const int grp = n / KS, ks = n % KS;
        const unsigned base = (grp < 2 ? ka : va) + b_off;
        if (grp % 2 == 0) ring[n % kSlots] = lds_read16_untracked<0>(base ^ (32u * ks));
        else ring[n % kSlots] = lds_read16_untracked<32 * D * 2>(base ^ (32u * ks));
      };
#pragma unroll
      for (int n = 0; n < kAhead; n++) issue(n);
#pragma unroll
      for (int n = 0; n < kItems; n++) {
        if (n + kAhead < kItems) issue(n + kAhead);
        wait_lgkmcnt(n + kAhead < kItems ? kAhead : kItems - 1 - n);
        settle(ring[n % kSlots]);
        const bf16x8 a = __builtin_bit_cast(bf16x8, ring[n % kSlots]);
        const int grp = n / KS, ks = n % KS;
        if (grp < 2) sacc[grp] = mfma_bf16(a, qf[ks], sacc[grp]);
        else dpacc[grp - 2] = mfma_bf16(a, gof[ks], dpacc[grp - 2]);
      }
    }
    // dS^T = P^T (.) (alpha dP^T - D^s), as B-operand fragments in token order
    bf16x8 dsf[4];
#pragma unroll
    for (int mt = 0; mt < 2; mt++)
#pragma unroll
      for (int e = 0; e < 16; e++) {
        float arg = sacc[mt][e] * c0 - L2;
        if (valid < kTileTokens) arg = 32 * mt + 8 * (e / 4) + 4 * g + e % 4 >= valid ? -INFINITY : arg;
        const float dsv = fast_exp2(arg) * (al * dpacc[mt][e] - Ds);
        sumds += dsv;
        dsf[2 * mt + e / 8][e % 8] = (__bf16)dsv;
      }
    // dQ^T += K^T dS^T: transposing reads of the K tile, those of the next 16-token step in flight
    // while the products of this one run
    {
      constexpr int kReads = 2 * ET;
      u32x2 rk[2][ET][2];
      auto issue = [&](int ks, int slot) {
#pragma unroll
        for (int et = 0; et < ET; et++)
#pragma unroll
          for (int hi = 0; hi < 2; hi++) rk[slot][et][hi] = lds_read_tr_untracked_at<16 * D>(ka + a_off[et], 2 * ks + hi);
      };
      issue(0, 0);
#pragma unroll
      for (int ks = 0; ks < kTileTokens / 16; ks++) {
        const int slot = ks & 1;
        if (ks + 1 < kTileTokens / 16) issue(ks + 1, slot ^ 1);
        wait_lgkmcnt(ks + 1 < kTileTokens / 16 ? kReads : 0);
#pragma unroll
        for (int et = 0; et < ET; et++) {
          settle(rk[slot][et][0]);
          settle(rk[slot][et][1]);
          const u32x4 v4 = {rk[slot][et][0][0], rk[slot][et][0][1], rk[slot][et][1][0], rk[slot][et][1][1]};
          dqacc[et] = mfma_bf16(__builtin_bit_cast(bf16x8, v4), dsf[ks], dqacc[et]);
        }
      }
    }
    __builtin_amdgcn_s_waitcnt(kVmcnt0);             // the next tile has landed in LDS ...
    __syncthreads();                                 // ... for everyone, and this tile's buffer is free
  }

  // ================= epilogue =================
  uint16_t* ta = reinterpret_cast<uint16_t*>(smem);                 // H_i^T [e][c]; then the dQ tile; then dO [row][e]
  uint16_t* tb = reinterpret_cast<uint16_t*>(smem + SM::kEpiA);     // w = Q^phi / (Q^phi Z_i) as [row][c]
  // dS K' = dS K - rowsum(dS) colmean(K)^T
  sumds = half_sum(sumds);
#pragma unroll
  for (int et = 0; et < ET; et++)
#pragma unroll
    for (int v4 = 0; v4 < 4; v4++) {
      const f32x4 m = *reinterpret_cast<const f32x4*>(mus + 32 * et + 8 * v4 + 4 * g);
#pragma unroll
      for (int r = 0; r < 4; r++) dqacc[et][4 * v4 + r] = (dqacc[et][4 * v4 + r] - sumds * m[r]) * rscale;
    }
  {
    const uint16_t* hsrc = h_i + slot * D * D;
    for (int idx = tid; idx < D * (D / 8); idx += NT) {
      const int e = idx / (D / 8), ch = idx % (D / 8);
      *reinterpret_cast<u32x4*>(ta + e * LD + 8 * ch) = *reinterpret_cast<const u32x4*>(hsrc + e * D + 8 * ch);
    }
    if (tid < D) zs[tid] = z_i[slot * D + tid];
  }
  // Q^phi = softmax_d(Q) of this lane's row from the Q fragments (channels 16 ks + 8 g + 0..7); the
  // fragments are overwritten with exp(q - max), the normalisation is applied where they are used
  // (the fragments are made opaque first: the widened copies that the prologue made of them would
  // otherwise be kept alive across the whole main loop for reuse here)
#pragma unroll
  for (int ks = 0; ks < KS; ks++) settle(qf[ks]);
  float qm = -INFINITY;
#pragma unroll
  for (int ks = 0; ks < KS; ks++)
#pragma unroll
    for (int e = 0; e < 8; e++) qm = fmaxf(qm, (float)qf[ks][e]);
  qm = half_max(qm);
  float qs = 0.f;
#pragma unroll
  for (int ks = 0; ks < KS; ks++)
#pragma unroll
    for (int e = 0; e < 8; e++) {
      const float x = fast_exp2(((float)qf[ks][e] - qm) * kLog2e);
      qs += x;
      qf[ks][e] = (__bf16)x;
    }
  qs = half_sum(qs);
  const float qinv = 1.f / qs;
  __syncthreads();                                   // H_i^T and Z_i visible
  float den = 0.f;
#pragma unroll
  for (int ks = 0; ks < KS; ks++) {
    const f32x4 z0 = *reinterpret_cast<const f32x4*>(zs + 16 * ks + 8 * g);
    const f32x4 z1 = *reinterpret_cast<const f32x4*>(zs + 16 * ks + 8 * g + 4);
#pragma unroll
    for (int e = 0; e < 8; e++) den += (float)qf[ks][e] * (e < 4 ? z0[e] : z1[e - 4]);
  }
  den = half_sum(den) * qinv;
  // every block selected: the linear branch receives and passes no gradient
  const float inv_den = (ksel >= Tn || !row_ok) ? 0.f : 1.f / den;
  // w as a [row][c] tile (zero rows past the end); the softmax-backward step reads Q^phi = w den back
  // from it in the layout of the accumulators
  {
    const float wscale = qinv * inv_den;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      bf16x8 wv;
#pragma unroll
      for (int e = 0; e < 8; e++) wv[e] = (__bf16)((float)qf[ks][e] * wscale);
      *reinterpret_cast<bf16x8*>(tb + qrow * LD + 16 * ks + 8 * g) = wv;
    }
  }
  // dQ^phi^T = (1 - alpha) H_i dO^T: A = H_i read transposed out of the H_i^T tile, B = the dO fragments
  f32x16 dqp[ET];
#pragma unroll
  for (int ct = 0; ct < ET; ct++)
#pragma unroll
    for (int e = 0; e < 16; e++) dqp[ct][e] = 0.f;
#pragma unroll
  for (int ks = 0; ks < KS; ks++)
#pragma unroll
    for (int ct = 0; ct < ET; ct++) dqp[ct] = mfma_bf16(nat_fragment<PL>(ta, ks, 32 * ct, lane), gof[ks], dqp[ct]);
  __syncthreads();                                   // w complete; nobody reads H_i^T any more
  // O^l is not kept by the forward pass: dO . O^l of a row equals sum_c w[r][c] (H_i dO^T)[c][r], both at
  // hand.  D^l = (1 - alpha) dO . O^l; the row's part of d alpha is dO . (O^s - O^l).
  float dot_l = 0.f;
#pragma unroll
  for (int ct = 0; ct < ET; ct++)
#pragma unroll
    for (int v4 = 0; v4 < 4; v4++) {
      const bf16x4 wq = *reinterpret_cast<const bf16x4*>(tb + qrow * LD + 32 * ct + 8 * v4 + 4 * g);
#pragma unroll
      for (int r = 0; r < 4; r++) dot_l += (float)wq[r] * dqp[ct][4 * v4 + r];
    }
  dot_l = half_sum(dot_l);
  const float Dl = (1.f - al) * dot_l;
  if (g == 0) dls[qrow] = Dl;
  {
    float mix = (row_ok && g == 0) ? dot_s - dot_l : 0.f;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) mix += __shfl_xor(mix, o);
    if (lane == 0) red[w] = mix;
  }
  float dot = 0.f;
#pragma unroll
  for (int ct = 0; ct < ET; ct++)
#pragma unroll
    for (int v4 = 0; v4 < 4; v4++) {
      const f32x4 z = *reinterpret_cast<const f32x4*>(zs + 32 * ct + 8 * v4 + 4 * g);
      const bf16x4 wq = *reinterpret_cast<const bf16x4*>(tb + qrow * LD + 32 * ct + 8 * v4 + 4 * g);
#pragma unroll
      for (int r = 0; r < 4; r++) {
        dqp[ct][4 * v4 + r] = ((1.f - al) * dqp[ct][4 * v4 + r] - Dl * z[r]) * inv_den;
        dot += dqp[ct][4 * v4 + r] * ((float)wq[r] * den);
      }
    }
  dot = half_sum(dot);
  // dQ = sparse part + softmax-backward(dQ^phi); transposed through LDS for a coalesced store
#pragma unroll
  for (int et = 0; et < ET; et++)
#pragma unroll
    for (int v4 = 0; v4 < 4; v4++) {
      const bf16x4 wq = *reinterpret_cast<const bf16x4*>(tb + qrow * LD + 32 * et + 8 * v4 + 4 * g);
      bf16x4 pk;
#pragma unroll
      for (int r = 0; r < 4; r++)
        pk[r] = (__bf16)(dqacc[et][4 * v4 + r] + (float)wq[r] * den * (dqp[et][4 * v4 + r] - dot));
      *reinterpret_cast<bf16x4*>(ta + qrow * LD + 32 * et + 8 * v4 + 4 * g) = pk;
    }
  __syncthreads();                                   // dQ tile complete; the waves' d alpha parts are visible
  if (tid == 0) {
    float t = 0.f;
#pragma unroll
    for (int x = 0; x < NW; x++) t += red[x];
    dalpha_part[slot] = t;
  }
  {
    uint16_t* dst = dq + head_offset(sin, bh, H) + (size_t)row0 * tok_stride;
    for (int idx = tid; idx < BQ * (D / 8); idx += NT) {
      const int r = idx / (D / 8), ch = idx % (D / 8);
      if (r < rows_valid)
        *reinterpret_cast<u32x4*>(dst + (size_t)r * tok_stride + 8 * ch) = *reinterpret_cast<const u32x4*>(ta + r * LD + 8 * ch);
    }
  }
  __syncthreads();                                   // the dQ tile has been read out
#pragma unroll
  for (int ks = 0; ks < KS; ks++) *reinterpret_cast<bf16x8*>(ta + qrow * LD + 16 * ks + 8 * g) = gof[ks];   // dO as [row][e]
  __syncthreads();
  // dH_i[c][e] = (1 - alpha) sum_r w[r][c] dO[r][e]: both operands read transposed, contraction over the rows
  constexpr int kTilesPerWave = ET * ET / NW;
  static_assert(kTilesPerWave >= 1, "unsupported split");
  uint16_t* dh_slot = dh_out + slot * D * D;
#pragma unroll 1
  for (int x = 0; x < kTilesPerWave; x++) {
    const int t = w * kTilesPerWave + x, ct = t / ET, et = t % ET;
    f32x16 acc;
#pragma unroll
    for (int e = 0; e < 16; e++) acc[e] = 0.f;
#pragma unroll
    for (int ks = 0; ks < BQ / 16; ks++)
      acc = mfma_bf16(v_fragment<PL>(tb, ks, 32 * ct, lane), v_fragment<PL>(ta, ks, 32 * et, lane), acc);
#pragma unroll
    for (int e = 0; e < 16; e++)
      dh_slot[(32 * ct + 8 * (e / 4) + 4 * g + e % 4) * D + 32 * et + lane % 32] = f32_to_bf16_bits((1.f - al) * acc[e]);
  }
  if (tid < D) {                                     // dZ_i[c] = -sum_r w[r][c] D^l_r
    float dz = 0.f;
    for (int r = 0; r < BQ; r++) dz -= bf16_bits_to_f32(tb[r * LD + tid]) * dls[r];
    dz_out[slot * D + tid] = dz;
  }
}

template <int D, int BQ>
static hipError_t launch_bwd_q_mfma(const Shape& s, const BwdArgs& a, hipStream_t stream) {
  constexpr int smem = BwdQSmem<D, BQ>::kBytes;
  static OncePerDevice once;
  if (hipError_t e = allow_dynamic_lds(once, (const void*)bwd_q_mfma_kernel<D, BQ>, smem); e != hipSuccess) return e;
  const int grid = ((s.Tm + kXcds - 1) / kXcds) * kXcds * s.BH;
  bwd_q_mfma_kernel<D, BQ><<<dim3((unsigned)grid), BQ * 2, smem, stream>>>(
      (const uint16_t*)a.q, (const uint16_t*)a.k, (const uint16_t*)a.v, (const uint16_t*)a.dout, (const uint16_t*)a.o_s,
      a.lse, a.k_mean, a.h_i, a.z_i, a.block_idx, a.alpha, (uint16_t*)a.dq, a.ds, a.lraw,
      (uint16_t*)a.dh, a.dz, a.dalpha_part, s.sin, s.sout, s.H, s.N, s.Tm, s.Tn, s.k, s.alpha_per_block ? 1 : 0);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
template <int D> struct BwdKvSmem {
  static constexpr int kLd = D + 8;
  static constexpr int kTile = SwizzledLayout<D>::kTileBytes;                  // one 64 x D bf16 tile
  static constexpr int kStepBytes = 4 * kTile;                                 // two buffers of (Q rows, dO rows);
                                                                               // after the loop: dH and K^phi, then the outputs
  static constexpr int kStatOff = kStepBytes;                                  // float [2][2][64]: L log2(e) and D^s of a step's rows
  static constexpr int kMuOff = kStatOff + 2 * 2 * 64 * 4;                     // float [D]  colmean(K)
  static constexpr int kDzOff = kMuOff + D * 4;                                // float [D]  dZ of this key block
  static constexpr int kDotOff = kDzOff + D * 4;                               // float [D / 32][64]
  static constexpr int kBytes = kDotOff + (D / 32) * 64 * 4;
  static_assert((D + 64) * kLd * 2 <= kStepBytes && 2 * 64 * kLd * 2 <= kStepBytes, "epilogue tiles reuse the step buffers");
};

// Scores are computed as S = Q K^T (query rows x keys) here: a lane of the result then owns one key
// and 16 of the 32 query rows of the tile, which is the B-operand layout of the products that contract
// over query rows (dV^T += dO^T P, dK^T += Q^T dS) - P and dS never leave registers.  Wave w owns the
// key half kh = w % 2 and the channel tiles of group w / 2; it computes the scores of all 64 rows of a
// step against its 32 keys (the two waves of a key half repeat that work: cheaper than passing P and dS
// through LDS with a barrier in between).  K_j and V_j live in registers as operand fragments.
template <int D, int BQ>
__global__ __launch_bounds__(256, 2) void bwd_kv_mfma_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const uint16_t* __restrict__ dout, const float* __restrict__ lraw2, const float* __restrict__ ds_in,
    const double* __restrict__ k_mean, const float* __restrict__ k_stats, const int32_t* __restrict__ col_ptr,
    const int32_t* __restrict__ col_idx, const uint16_t* __restrict__ dh_in, const float* __restrict__ dz_in,
    const float* __restrict__ dh_total, const float* __restrict__ dz_total, const float* __restrict__ alpha,
    uint16_t* __restrict__ dk, uint16_t* __restrict__ dv, float* __restrict__ colsum, Strides sin, Strides sout, int H,
    int N, int Tm, int Tn, int ksel, int alpha_per_block) {
  constexpr int NW = 4, NT = 256;
  constexpr int LD = D + 8, KS = D / 16, ET = D / 32;
  constexpr int HP = BQ / 64;                        // 64-row steps per query block
  constexpr int CT = ET / 2;                         // 32-channel tiles of dV^T / dK^T per wave
  typedef SwizzledLayout<D> SL;
  typedef PaddedLayout<D> PL;
  typedef BwdKvSmem<D> SM;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  auto qbuf = [&](int buf) { return reinterpret_cast<uint16_t*>(smem + buf * 2 * SM::kTile); };
  auto gbuf = [&](int buf) { return reinterpret_cast<uint16_t*>(smem + buf * 2 * SM::kTile + SM::kTile); };
  float* stat = reinterpret_cast<float*>(smem + SM::kStatOff);
  float* mus = reinterpret_cast<float*>(smem + SM::kMuOff);
  float* dzs = reinterpret_cast<float*>(smem + SM::kDzOff);
  float* dred = reinterpret_cast<float*>(smem + SM::kDotOff);

  // the same dealing for key blocks: 8 runs of consecutive key blocks per head, one per XCD
  const int per_head = (Tn + kXcds - 1) / kXcds;
  const int bh = (blockIdx.x / kXcds) / per_head, j = (blockIdx.x % kXcds) * per_head + (blockIdx.x / kXcds) % per_head;
  if (j >= Tn) return;
  const int h = bh % H;
  const int tid = threadIdx.x, lane = tid % kWave, g = lane / 32;
  const int w = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int kh = w & 1, cgrp = w >> 1;
  const int t0 = j * kTileTokens, valid = min(kTileTokens, N - t0);
  const int mykey = 32 * kh + lane % 32;             // this lane's key inside the block
  const bool key_ok = mykey < valid;
  const uint16_t* qh = q + head_offset(sin, bh, H);
  const uint16_t* kh_ = k + head_offset(sin, bh, H);
  const uint16_t* vh = v + head_offset(sin, bh, H);
  const uint16_t* doh = dout + head_offset(sout, bh, H);
  const int tok_stride = sin.n;
  const float rscale = rsqrtf((float)D);
  const float c0 = kLog2e * rscale;

  // K_j and V_j rows of this lane's key as operand fragments (rows past the end repeat the last one)
  bf16x8 kfr[KS], vfr[KS];
  {
    const size_t row = (size_t)(t0 + min(mykey, valid - 1)) * tok_stride + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      kfr[ks] = *reinterpret_cast<const bf16x8*>(kh_ + row + 16 * ks);
      vfr[ks] = *reinterpret_cast<const bf16x8*>(vh + row + 16 * ks);
    }
  }
  if (tid < D) mus[tid] = (float)k_mean[(size_t)bh * D + tid];

  const int32_t* cp = col_ptr + (size_t)bh * (Tn + 1);
  const int32_t* ci = col_idx + (size_t)bh * Tm * ksel;
  const int l0 = __builtin_amdgcn_readfirstlane(cp[j]), l1 = __builtin_amdgcn_readfirstlane(cp[j + 1]);
  const int nsteps = (l1 - l0) * HP;

  // Step t covers rows [64 (t % HP), +64) of query block ci[l0 + t / HP].  A half block with no rows
  // (short last query block) still runs, on the block's first rows with every probability masked.
  // The rows of step t + 1 (and L log2 e, D^s of those rows) are requested at the start of step t,
  // straight into LDS; the query block index is read one step before that.
  struct Step { int rows, src0; float al; };
  auto block_of = [&](int t) { return ci[l0 + min(t, nsteps - 1) / HP]; };
  auto place = [&](int t, int i) {
    Step st;
    const int row0 = i * BQ + 64 * (t % HP);
    st.rows = max(0, min(64, N - row0));
    st.src0 = st.rows > 0 ? row0 : i * BQ;
    st.al = alpha[alpha_per_block ? (size_t)h * Tm + i : (size_t)h];
    return st;
  };
  auto request = [&](const Step& st, int buf) {
    const int dma_rows = max(st.rows, 1);
    dma_tile<D, NW>(qh + (size_t)st.src0 * tok_stride, tok_stride, dma_rows, qbuf(buf), w, lane);
    dma_tile<D, NW>(doh + (size_t)st.src0 * sout.n, sout.n, dma_rows, gbuf(buf), w, lane);
    // every wave fetches the same 2 x 64 floats (same values to the same place: the counts of
    // outstanding transfers stay equal across the waves)
    const size_t at = (size_t)bh * N + st.src0 + min(lane, dma_rows - 1);
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(lraw2 + at),
                                     (__attribute__((address_space(3))) void*)(stat + buf * 128), 4, 0, 0);
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(ds_in + at),
                                     (__attribute__((address_space(3))) void*)(stat + buf * 128 + 64), 4, 0, 0);
  };

  f32x16 dvacc[CT], dkacc[CT];
#pragma unroll
  for (int x = 0; x < CT; x++)
#pragma unroll
    for (int e = 0; e < 16; e++) { dvacc[x][e] = 0.f; dkacc[x][e] = 0.f; }

  Step cur{0, 0, 0.f};
  int i_nxt = 0;
  if (nsteps > 0) {
    cur = place(0, block_of(0));
    i_nxt = block_of(1);
    request(cur, 0);
  }
  wait_vmcnt<0>();
#pragma unroll
  for (int ks = 0; ks < KS; ks++) { settle(kfr[ks]); settle(vfr[ks]); }
  __syncthreads();                                   // step 0 and mus are in LDS for everyone

  // LDS byte offsets of this lane's operand reads inside a Q or dO tile.  Row-wise reads: row
  // l % 32 (+ 32 for the second row half), channel step ks at (offset of step 0) ^ 32 ks.
  // Transposing reads (cf. read_tr4): the row swizzle depends on row % 8 only, so 16-row step ks
  // sits at a fixed distance from step 0.
  const unsigned b_off = (unsigned)SL::offset(lane % 32, 8 * g) * 2;
  const int tr_row = 4 * g + (lane % 16) / 4, tr_col = 16 * ((lane / 16) % 2) + 4 * (lane % 4);
  unsigned a_off[CT];
#pragma unroll
  for (int x = 0; x < CT; x++) a_off[x] = (unsigned)SL::offset(tr_row, 32 * (CT * cgrp + x) + tr_col) * 2;

  for (int t = 0; t < nsteps; t++) {
    const int buf = t & 1;
    Step nxt = cur;
    if (t + 1 < nsteps) {
      nxt = place(t + 1, i_nxt);
      request(nxt, buf ^ 1);
    }
    i_nxt = block_of(t + 2);
    const unsigned qa = lds_address(qbuf(buf)), ga = lds_address(gbuf(buf));
    const float* st_l = stat + buf * 128;
    // S = Q K^T and dP = dO V^T: rows 32 rh.. x this wave's 32 keys.  32 operand reads (this lane's
    // rows of Q and dO), each feeding one product; 8 are kept in flight.
    f32x16 sacc[2], dpacc[2];
#pragma unroll
    for (int rh = 0; rh < 2; rh++)
#pragma unroll
      for (int e = 0; e < 16; e++) { sacc[rh][e] = 0.f; dpacc[rh][e] = 0.f; }
    {
      constexpr int kItems = 4 * KS, kAhead = 8, kSlots = kAhead + 1;
      u32x4 ring[kSlots];
      auto issue = [&](int n) {                      // item n: (Q | dO, row half, channel step)
        const int grp = n / KS, ks = n % KS;
        const unsigned base = (grp < 2 ? qa : ga) + b_off;
        if (grp % 2 == 0) ring[n % kSlots] = lds_read16_untracked<0>(base ^ (32u * ks));
        else ring[n % kSlots] = lds_read16_untracked<32 * D * 2>(base ^ (32u * ks));
      };
#pragma unroll
      for (int n = 0; n < kAhead; n++) issue(n);
#pragma unroll
      for (int n = 0; n < kItems; n++) {
        if (n + kAhead < kItems) issue(n + kAhead);
        wait_lgkmcnt(n + kAhead < kItems ? kAhead : kItems - 1 - n);
        settle(ring[n % kSlots]);
        const bf16x8 a = __builtin_bit_cast(bf16x8, ring[n % kSlots]);
        const int grp = n / KS, ks = n % KS;
        if (grp < 2) sacc[grp] = mfma_bf16(a, kfr[ks], sacc[grp]);
        else dpacc[grp - 2] = mfma_bf16(a, vfr[ks], dpacc[grp - 2]);
      }
    }
    // alpha P and dS = P (.) (alpha dP - D^s), as B-operand fragments over the 64 rows (token order);
    // masked entries get exp2(-inf) = 0
    bf16x8 pf[4], dsf[4];
    auto probabilities = [&](auto masked) {          // masked: a short key block or a short last row block
#pragma unroll
      for (int rh = 0; rh < 2; rh++)
#pragma unroll
        for (int v4 = 0; v4 < 4; v4++) {
          const f32x4 l4 = *reinterpret_cast<const f32x4*>(st_l + 32 * rh + 8 * v4 + 4 * g);
          const f32x4 d4 = *reinterpret_cast<const f32x4*>(st_l + 64 + 32 * rh + 8 * v4 + 4 * g);
#pragma unroll
          for (int r = 0; r < 4; r++) {
            float arg = sacc[rh][4 * v4 + r] * c0 - l4[r];
            if constexpr (decltype(masked)::value)
              arg = (!key_ok || 32 * rh + 8 * v4 + 4 * g + r >= cur.rows) ? -INFINITY : arg;
            const float p = fast_exp2(arg);
            pf[2 * rh + v4 / 2][4 * (v4 % 2) + r] = (__bf16)(cur.al * p);
            dsf[2 * rh + v4 / 2][4 * (v4 % 2) + r] = (__bf16)(p * (cur.al * dpacc[rh][4 * v4 + r] - d4[r]));
          }
        }
    };
    if (cur.rows < 64 || valid < kTileTokens) probabilities(std::true_type{});
    else probabilities(std::false_type{});
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // nothing tracked is in flight when the counted reads below start
    // dV^T += dO^T (alpha P), dK'^T += Q^T dS: contraction over the 64 rows of the step; the operand
    // reads of the next 16-row step are in flight while the products of this one run
    {
      constexpr int kReads = 4 * CT;
      u32x2 rg[2][CT][2], rq[2][CT][2];
      auto issue = [&](int ks, int slot) {
#pragma unroll
        for (int x = 0; x < CT; x++)
#pragma unroll
          for (int hi = 0; hi < 2; hi++) {
            rg[slot][x][hi] = lds_read_tr_untracked_at<16 * D>(ga + a_off[x], 2 * ks + hi);
            rq[slot][x][hi] = lds_read_tr_untracked_at<16 * D>(qa + a_off[x], 2 * ks + hi);
          }
      };
      auto frag = [&](u32x2 (&r)[2]) {
        settle(r[0]);
        settle(r[1]);
        const u32x4 v4 = {r[0][0], r[0][1], r[1][0], r[1][1]};
        return __builtin_bit_cast(bf16x8, v4);
      };
      issue(0, 0);
#pragma unroll
      for (int ks = 0; ks < 4; ks++) {
        const int slot = ks & 1;
        if (ks + 1 < 4) issue(ks + 1, slot ^ 1);
        wait_lgkmcnt(ks + 1 < 4 ? kReads : 0);
#pragma unroll
        for (int x = 0; x < CT; x++) {
          dvacc[x] = mfma_bf16(frag(rg[slot][x]), pf[ks], dvacc[x]);
          dkacc[x] = mfma_bf16(frag(rq[slot][x]), dsf[ks], dkacc[x]);
        }
      }
    }
    wait_vmcnt<0>();                                 // the next step's rows have landed ...
    asm volatile("s_barrier" ::: "memory");          // ... for everyone; this step's tiles are free
    cur = nxt;
  }
  __syncthreads();

  // ================= linear branch =================
  uint16_t* dht = reinterpret_cast<uint16_t*>(smem);                     // dH [c][e] as bf16, row stride LD
  uint16_t* kpt = dht + D * LD;                                          // K^phi_j [key][c], row stride LD
  const bool all_selected = ksel >= Tn;
  {
    // dH = dH_total - sum over the query blocks that selected j of dH_i (Alg. 3's M_c[i, j] = 0 sum)
    constexpr int NCH = D * D / 8 / NT;              // 16-byte chunks per thread
    float acc[NCH][8];
#pragma unroll
    for (int n = 0; n < NCH; n++) {
      const int idx = tid + NT * n;
      const float* tot = dh_total + (size_t)bh * D * D + (size_t)idx * 8;
      const f32x4 a = *reinterpret_cast<const f32x4*>(tot), b = *reinterpret_cast<const f32x4*>(tot + 4);
#pragma unroll
      for (int e = 0; e < 4; e++) { acc[n][e] = all_selected ? 0.f : a[e]; acc[n][4 + e] = all_selected ? 0.f : b[e]; }
    }
    float dzj = (tid < D && !all_selected) ? dz_total[(size_t)bh * D + tid] : 0.f;
    if (!all_selected)
      for (int l = l0; l < l1; l++) {
        const size_t slot = (size_t)bh * Tm + ci[l];
        const uint16_t* src = dh_in + slot * D * D;
#pragma unroll
        for (int n = 0; n < NCH; n++) {
          const bf16x8 x = *reinterpret_cast<const bf16x8*>(src + (size_t)(tid + NT * n) * 8);
#pragma unroll
          for (int e = 0; e < 8; e++) acc[n][e] -= (float)x[e];
        }
        if (tid < D) dzj -= dz_in[slot * D + tid];
      }
#pragma unroll
    for (int n = 0; n < NCH; n++) {
      const int idx = tid + NT * n, c = idx / (D / 8), ch = idx % (D / 8);
      bf16x8 y;
#pragma unroll
      for (int e = 0; e < 8; e++) y[e] = (__bf16)acc[n][e];
      *reinterpret_cast<bf16x8*>(dht + c * LD + 8 * ch) = y;
    }
    if (tid < D) dzs[tid] = dzj;
  }
  // K_j -> K^phi_j = exp(K - colmean(K) - lnZ) in the fragment registers (keys past the end: 0); one
  // wave of each key half also leaves it in LDS for the softmax-backward step
  {
    const float lnz2 = k_stats[(size_t)bh * N + t0 + min(mykey, valid - 1)] * kLog2e;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      const f32x4 m0 = *reinterpret_cast<const f32x4*>(mus + 16 * ks + 8 * g);
      const f32x4 m1 = *reinterpret_cast<const f32x4*>(mus + 16 * ks + 8 * g + 4);
#pragma unroll
      for (int e = 0; e < 8; e++) {
        const float kp = key_ok ? fast_exp2(((float)kfr[ks][e] - (e < 4 ? m0[e] : m1[e - 4])) * kLog2e - lnz2) : 0.f;
        kfr[ks][e] = (__bf16)kp;
      }
      if (cgrp == 0) *reinterpret_cast<bf16x8*>(kpt + mykey * LD + 16 * ks + 8 * g) = kfr[ks];
    }
  }
  __syncthreads();
  // dK^phi^T = dH V^T (+ dZ 1^T below) and dV^T += dH^T K^phi^T, both channels x keys; V_j and K^phi_j
  // are the B operands, from registers
  f32x16 dkp[CT];
#pragma unroll
  for (int x = 0; x < CT; x++)
#pragma unroll
    for (int e = 0; e < 16; e++) dkp[x][e] = 0.f;
#pragma unroll
  for (int ks = 0; ks < KS; ks++) {
#pragma unroll
    for (int x = 0; x < CT; x++) {
      const int ct = CT * cgrp + x;
      dkp[x] = mfma_bf16(row_fragment<PL>(dht, 32 * ct + lane % 32, 16 * ks + 8 * g), vfr[ks], dkp[x]);   // over e
      dvacc[x] = mfma_bf16(nat_fragment<PL>(dht, ks, 32 * ct, lane), kfr[ks], dvacc[x]);                 // over c
    }
  }
  // back through phi: dK' += K^phi (.) (dK^phi - rowsum(dK^phi (.) K^phi)); the row sum spans all channels
  float kp[CT][16];
#pragma unroll
  for (int x = 0; x < CT; x++) {
    const int ct = CT * cgrp + x;
    float part = 0.f;
#pragma unroll
    for (int v4 = 0; v4 < 4; v4++) {
      const bf16x4 kk = *reinterpret_cast<const bf16x4*>(kpt + mykey * LD + 32 * ct + 8 * v4 + 4 * g);
      const f32x4 dz = *reinterpret_cast<const f32x4*>(dzs + 32 * ct + 8 * v4 + 4 * g);
#pragma unroll
      for (int r = 0; r < 4; r++) {
        kp[x][4 * v4 + r] = (float)kk[r];
        dkp[x][4 * v4 + r] += dz[r];
        part += dkp[x][4 * v4 + r] * kp[x][4 * v4 + r];
      }
    }
    part = half_sum(part);
    if (g == 0) dred[ct * 64 + mykey] = part;
  }
  __syncthreads();                                   // row sums complete; every wave is done with the dH and K^phi tiles
  uint16_t* okt = dht;                               // dK' [key][c], then dV [key][e] behind it
  uint16_t* ovt = dht + 64 * LD;
  {
    float dot = 0.f;
#pragma unroll
    for (int c2 = 0; c2 < ET; c2++) dot += dred[c2 * 64 + mykey];
#pragma unroll
    for (int x = 0; x < CT; x++) {
      const int ct = CT * cgrp + x;
#pragma unroll
      for (int v4 = 0; v4 < 4; v4++) {
        bf16x4 pk, pv;
#pragma unroll
        for (int r = 0; r < 4; r++) {
          pk[r] = (__bf16)(dkacc[x][4 * v4 + r] * rscale + kp[x][4 * v4 + r] * (dkp[x][4 * v4 + r] - dot));
          pv[r] = (__bf16)dvacc[x][4 * v4 + r];
        }
        *reinterpret_cast<bf16x4*>(okt + mykey * LD + 32 * ct + 8 * v4 + 4 * g) = pk;
        *reinterpret_cast<bf16x4*>(ovt + mykey * LD + 32 * ct + 8 * v4 + 4 * g) = pv;
      }
    }
  }
  __syncthreads();
  {
    uint16_t* dkh = dk + head_offset(sin, bh, H) + (size_t)t0 * tok_stride;
    uint16_t* dvh = dv + head_offset(sin, bh, H) + (size_t)t0 * tok_stride;
    for (int idx = tid; idx < kTileTokens * (D / 8); idx += NT) {
      const int t = idx / (D / 8), ch = idx % (D / 8);
      if (t < valid) {
        *reinterpret_cast<u32x4*>(dkh + (size_t)t * tok_stride + 8 * ch) = *reinterpret_cast<const u32x4*>(okt + t * LD + 8 * ch);
        *reinterpret_cast<u32x4*>(dvh + (size_t)t * tok_stride + 8 * ch) = *reinterpret_cast<const u32x4*>(ovt + t * LD + 8 * ch);
      }
    }
    if (tid < D) {                                   // column sums of dK' (as stored) for the smoothing term
      float sum = 0.f;
      for (int t = 0; t < valid; t++) sum += bf16_bits_to_f32(okt[t * LD + tid]);
      colsum[((size_t)bh * Tn + j) * D + tid] = sum;
    }
  }
}

template <int D, int BQ>
static hipError_t launch_bwd_kv_mfma(const Shape& s, const BwdArgs& a, hipStream_t stream) {
  constexpr int smem = BwdKvSmem<D>::kBytes;
  static OncePerDevice once;
  if (hipError_t e = allow_dynamic_lds(once, (const void*)bwd_kv_mfma_kernel<D, BQ>, smem); e != hipSuccess) return e;
  const int grid = ((s.Tn + kXcds - 1) / kXcds) * kXcds * s.BH;
  bwd_kv_mfma_kernel<D, BQ><<<dim3((unsigned)grid), 256, smem, stream>>>(
      (const uint16_t*)a.q, (const uint16_t*)a.k, (const uint16_t*)a.v, (const uint16_t*)a.dout, a.lraw, a.ds, a.k_mean,
      a.k_stats, a.col_ptr, a.col_idx, (const uint16_t*)a.dh, a.dz, a.dh_total, a.dz_total, a.alpha, (uint16_t*)a.dk,
      (uint16_t*)a.dv, a.colsum, s.sin, s.sout, s.H, s.N, s.Tm, s.Tn, s.k, s.alpha_per_block ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch_bwd_kv_bf16(const Shape& s, const BwdArgs& a, hipStream_t stream) {
  if (s.d == 128 && s.bq == 128) return launch_bwd_kv_mfma<128, 128>(s, a, stream);
  if (s.d == 128 && s.bq == 64) return launch_bwd_kv_mfma<128, 64>(s, a, stream);
  if (s.d == 64 && s.bq == 128) return launch_bwd_kv_mfma<64, 128>(s, a, stream);
  return launch_bwd_kv_mfma<64, 64>(s, a, stream);
}

hipError_t launch_bwd_q_bf16(const Shape& s, const BwdArgs& a, hipStream_t stream) {
  if (s.d == 128 && s.bq == 128) return launch_bwd_q_mfma<128, 128>(s, a, stream);
  if (s.d == 128 && s.bq == 64) return launch_bwd_q_mfma<128, 64>(s, a, stream);
  if (s.d == 64 && s.bq == 128) return launch_bwd_q_mfma<64, 128>(s, a, stream);
  return launch_bwd_q_mfma<64, 64>(s, a, stream);
}

}  // namespace sla2
