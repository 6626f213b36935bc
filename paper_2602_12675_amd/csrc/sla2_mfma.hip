// bf16 / FP8 path of the SLA2 forward pass on the gfx950 matrix cores (Alg. 2 of the paper).
//
//   kv_state_bf16   per key block j of a head: K^phi_j = softmax_d(K_j - colmean K), written out as bf16
//                   MFMA operand fragments; z_j = colsum(K^phi_j); per-chunk partial sums of
//                   h_j = (K^phi_j)^T V_j and z_j (reduced to the per-head totals by kv_total); in the
//                   low-bit modes also the e4m3 or INT8 codes of K - colmean K with one scale per key
//                   block, and, when V is quantised too, the e4m3 codes of V in operand order (Sec. 5).
//   attn_mfma       one workgroup per query block i:
//                     sparse branch over the selected key/value blocks, ascending (online softmax);
//                     the d x d state of exactly those blocks, sum_sel (K^phi_j)^T V_j, from the stored
//                     K^phi fragments and the V tile that is already staged for P V;
//                     H_i = H_total - that sum, Z_i = Z_total - sum_sel z_j  (complement of the
//                     M_c[i,j] = 0 sum of Alg. 2);  O_l = Q^phi H_i / (Q^phi Z_i);
//                     out = alpha O_s + (1 - alpha) O_l                                     (Eq. 13)
//                   The same kernel with the block list replaced by 0..T_n-1 and the linear branch
//                   compiled out is the dense attention comparator.
//
// Products run as v_mfma_f32_32x32x16_bf16 with fp32 accumulation.  In the low-bit modes (Sec. 5) Q K^T
// runs on 8-bit codes: 64-deep v_mfma_f32_32x32x64_f8f6f4 (e4m3) or 32-deep v_mfma_i32_32x32x32_i8 (INT8);
// with V quantised as well, P V is a 64-deep FP8 product too.  Scores are kept transposed (S^T = K Q^T) so that one lane owns one query row:
// row maxima and sums are in-lane reductions plus one exchange between the two lane halves, and
// the probabilities go back into the next product as its B operand without leaving registers.
#include "mfma_tiles.h"

namespace sla2 {

// four values already scaled into [-127, 127] -> their nearest integers (ties to even), one per byte
__device__ __forceinline__ int pack_int8(float a, float b, float c, float d) {
  const int ia = (int)__builtin_rintf(a), ib = (int)__builtin_rintf(b), ic = (int)__builtin_rintf(c), id = (int)__builtin_rintf(d);
  return (ia & 0xff) | ((ib & 0xff) << 8) | ((ic & 0xff) << 16) | (id << 24);
}

// How the (D/32)^2 32x32 tiles of the d x d state h are spread over NW waves: wave w owns
// kMtw x kNtw tiles starting at (mt0, nt0).
template <int D, int NW> struct HSplit {
  static constexpr int kMt = D / 32;
  static constexpr int kPerWave = kMt * kMt / NW;
  static constexpr int kMtw = kPerWave > kMt ? kPerWave / kMt : 1;
  static constexpr int kNtw = kPerWave / kMtw;
  static_assert(kPerWave >= 1 && kMtw * kNtw == kPerWave, "unsupported split");
  __device__ static int mt0(int w) { return (w * kPerWave) / kMt; }
  __device__ static int nt0(int w) { return (w * kPerWave) % kMt; }
};

// K^phi of one key block is stored as the A-operand fragments of the product K^phi^T V:
// [block][mt = channel tile][ks = 16-token step][lane][8 bf16], lane l holding channel 32 mt + l % 32
// and the 8 tokens of (ks, l / 32) in token order - 1 KB per fragment, read back with one
// coalesced 16-byte load per lane and no LDS traffic.
template <int D>
__device__ __forceinline__ size_t kphi_offset(size_t block, int mt, int ks, int lane) {
  return (((block * (D / 32) + mt) * (kTileTokens / 16) + ks) * kWave + lane) * 8;
}

// =============================================================================================
// kv_state_bf16
// =============================================================================================
template <int D, int QUANT>   // QUANT: 0 none, 1 FP8 e4m3 codes of K - colmean K, 2 INT8 codes, 3 as 1 plus e4m3 codes of V
__global__ __launch_bounds__(256) void kv_state_bf16_kernel(const uint16_t* __restrict__ k,
                                                            const uint16_t* __restrict__ v,
                                                            const double* __restrict__ k_mean,
                                                            float* __restrict__ k_stats, float* __restrict__ partial,
                                                            uint16_t* __restrict__ k_phi, float* __restrict__ z_blocks,
                                                            uint8_t* __restrict__ k_codes, float* __restrict__ k_scale,
                                                            uint8_t* __restrict__ v_codes, float* __restrict__ v_scale,
                                                            Strides sin, int H, int N, int Tn, int chunks,
                                                            int blocks_per_chunk) {
  constexpr int LD = TileGeom<D>::kLd;
  typedef HSplit<D, 4> HS;
  __shared__ __attribute__((aligned(16))) uint16_t ktile[kTileTokens * LD];
  __shared__ __attribute__((aligned(16))) uint16_t vtile[kTileTokens * LD];
  __shared__ __attribute__((aligned(16))) float lnz2[kTileTokens];
  __shared__ float mu_s[D];
  __shared__ float red[4];
  __shared__ float red_v[4];
  const int bh = blockIdx.x / chunks, chunk = blockIdx.x % chunks;
  const int tid = threadIdx.x, lane = tid % kWave, w = tid / kWave, g = lane / 32;
  const uint16_t* kh = k + head_offset(sin, bh, H);
  const uint16_t* vh = v + head_offset(sin, bh, H);
  const int j0 = chunk * blocks_per_chunk, j1 = min(Tn, j0 + blocks_per_chunk);
  const int mt0 = HS::mt0(w), nt0 = HS::nt0(w);

  if (tid < D) mu_s[tid] = (float)k_mean[(size_t)bh * D + tid];
  __syncthreads();
  float mu2[HS::kMtw];
#pragma unroll
  for (int a = 0; a < HS::kMtw; a++) mu2[a] = mu_s[32 * (mt0 + a) + lane % 32] * kLog2e;

  f32x16 hacc[HS::kMtw][HS::kNtw];
  float zacc[HS::kMtw];
#pragma unroll
  for (int a = 0; a < HS::kMtw; a++) {
    zacc[a] = 0.f;
#pragma unroll
    for (int b = 0; b < HS::kNtw; b++)
#pragma unroll
      for (int e = 0; e < 16; e++) hacc[a][b][e] = 0.f;
  }

  typedef TileCopy<D, 256> TC;
  u32x4 kr[TC::kLoads], vr[TC::kLoads];
  if (j0 < j1) {
    const int valid = min(kTileTokens, N - j0 * kTileTokens);
    TC::load(kr, kh + (size_t)j0 * kTileTokens * sin.n, sin.n, valid, tid);
    TC::load(vr, vh + (size_t)j0 * kTileTokens * sin.n, sin.n, valid, tid);
  }
  for (int j = j0; j < j1; j++) {
    const int t0 = j * kTileTokens, valid = min(kTileTokens, N - t0);
    __syncthreads();                                   // previous tile fully consumed
    TC::store(kr, ktile, tid);
    TC::store(vr, vtile, tid);
    if (j + 1 < j1) {
      const int nvalid = min(kTileTokens, N - (j + 1) * kTileTokens);
      TC::load(kr, kh + (size_t)(j + 1) * kTileTokens * sin.n, sin.n, nvalid, tid);
      TC::load(vr, vh + (size_t)(j + 1) * kTileTokens * sin.n, sin.n, nvalid, tid);
    }
    __syncthreads();
    {  // per-token log-partition of softmax_d(k'), 4 threads per token
      const int t = tid / 4, sub = tid % 4;
      float x[D / 4];
      float m = -INFINITY, amax = 0.f;
#pragma unroll
      for (int i = 0; i < D / 32; i++) {
        const int c0 = 8 * (sub + 4 * i);
        uint4 u = *reinterpret_cast<const uint4*>(ktile + t * LD + c0);
        uint32_t wds[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int e = 0; e < 4; e++) {
          x[8 * i + 2 * e] = __builtin_bit_cast(float, wds[e] << 16) - mu_s[c0 + 2 * e];
          x[8 * i + 2 * e + 1] = __builtin_bit_cast(float, wds[e] & 0xFFFF0000u) - mu_s[c0 + 2 * e + 1];
        }
      }
#pragma unroll
      for (int i = 0; i < D / 4; i++) { m = fmaxf(m, x[i]); amax = fmaxf(amax, fabsf(x[i])); }
      m = fmaxf(m, __shfl_xor(m, 1));
      m = fmaxf(m, __shfl_xor(m, 2));
      float sum = 0.f;
#pragma unroll
      for (int i = 0; i < D / 4; i++) sum += fast_exp2((x[i] - m) * kLog2e);
      sum += __shfl_xor(sum, 1);
      sum += __shfl_xor(sum, 2);
      const float lnz = m + __log2f(sum) * 0.6931471805599453f;
      const bool ok = t < valid;
      if (sub == 0) {
        lnz2[t] = ok ? lnz * kLog2e : INFINITY;
        if (ok) k_stats[(size_t)bh * N + t0 + t] = lnz;
      }
      if (QUANT) {
        // one scale per key block: amax over the block's existing tokens (Sec. 5; see sla2.h)
        constexpr float kCodeMax = QUANT == 2 ? kInt8Max : kE4M3Max;
        if (!ok) amax = 0.f;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) amax = fmaxf(amax, __shfl_xor(amax, o));
        if (lane == 0) red[w] = amax;
        __syncthreads();
        amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        const float inv = amax > 0.f ? kCodeMax / amax : 1.f;
        if (tid == 0) k_scale[(size_t)bh * Tn + j] = amax > 0.f ? amax / kCodeMax : 1.f;
        uint8_t* dst = k_codes + (((size_t)bh * Tn + j) * kTileTokens + t) * D;
#pragma unroll
        for (int i = 0; i < D / 32; i++) {
          const int c0 = 8 * (sub + 4 * i);
          int lo = 0, hi = 0;
          if (ok) {
            float y[8];
#pragma unroll
            for (int e = 0; e < 8; e++) y[e] = fminf(fmaxf(x[8 * i + e] * inv, -kCodeMax), kCodeMax);
            if constexpr (QUANT == 2) {
              lo = pack_int8(y[0], y[1], y[2], y[3]);
              hi = pack_int8(y[4], y[5], y[6], y[7]);
            } else {
              lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], lo, false);
              lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], lo, true);
              hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[4], y[5], hi, false);
              hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[6], y[7], hi, true);
            }
          }
          *reinterpret_cast<int2*>(dst + c0) = make_int2(lo, hi);
        }
      }
    }
    if constexpr (QUANT == 3) {
      // quant(V_j) for the second product (Alg. 2): one e4m3 scale per block over its existing tokens,
      // codes stored channel-major with the tokens of a row in the order the 64-deep product consumes
      // them (layout: sla2.h, v_fp8).  Thread (token t, quarter sub) finds the maximum ...
      const int t = tid / 4, sub = tid % 4;
      float vmax = 0.f;
      if (t < valid) {
#pragma unroll
        for (int i = 0; i < D / 32; i++) {
          const uint4 u = *reinterpret_cast<const uint4*>(vtile + t * LD + 8 * (sub + 4 * i));
          const uint32_t wds[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
          for (int e = 0; e < 4; e++) {
            vmax = fmaxf(vmax, fabsf(__builtin_bit_cast(float, wds[e] << 16)));
            vmax = fmaxf(vmax, fabsf(__builtin_bit_cast(float, wds[e] & 0xFFFF0000u)));
          }
        }
      }
#pragma unroll
      for (int o = 1; o < kWave; o <<= 1) vmax = fmaxf(vmax, __shfl_xor(vmax, o));
      if (lane == 0) red_v[w] = vmax;
      __syncthreads();
      vmax = fmaxf(fmaxf(red_v[0], red_v[1]), fmaxf(red_v[2], red_v[3]));
      const float vinv = vmax > 0.f ? kE4M3Max / vmax : 1.f;
      if (tid == 0) v_scale[(size_t)bh * Tn + j] = vmax > 0.f ? vmax / kE4M3Max : 1.f;
      // ... and thread (channel c, half gh) writes the 32 codes of bytes 32 gh .. 32 gh + 31 of row c
      if (tid < 2 * D) {
        const int c = tid / 2, gh = tid % 2;
        int wd[8];
#pragma unroll
        for (int q = 0; q < 8; q++) {                  // dword q = bytes 4 q .. 4 q + 3
          float y[4];
#pragma unroll
          for (int r = 0; r < 4; r++) {
            const int b = 4 * q + r;
            const int tok = 32 * (b / 16) + 8 * ((b % 16) / 4) + 4 * gh + b % 4;
            const float x = __builtin_bit_cast(float, (uint32_t)vtile[tok * LD + c] << 16);
            y[r] = tok < valid ? fminf(fmaxf(x * vinv, -kE4M3Max), kE4M3Max) : 0.f;
          }
          int d0 = 0;
          d0 = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], d0, false);
          d0 = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], d0, true);
          wd[q] = d0;
        }
        int4* dst = reinterpret_cast<int4*>(v_codes + (((size_t)bh * Tn + j) * D + c) * kTileTokens + 32 * gh);
        dst[0] = make_int4(wd[0], wd[1], wd[2], wd[3]);
        dst[1] = make_int4(wd[4], wd[5], wd[6], wd[7]);
      }
    }
    __syncthreads();
    // K^phi fragments (kept for the attention kernel), h += K^phi^T V on the matrix cores, z_j
    float zsum[HS::kMtw];
#pragma unroll
    for (int a = 0; a < HS::kMtw; a++) zsum[a] = 0.f;
#pragma unroll
    for (int ks = 0; ks < kTileTokens / 16; ks++) {
      bf16x8 kf[HS::kMtw];
#pragma unroll
      for (int a = 0; a < HS::kMtw; a++) {
        kf[a] = kphi_fragment<PaddedLayout<D>>(ktile, lnz2, mu2[a], ks, 32 * (mt0 + a), lane, zsum[a]);
        if (nt0 == 0)
          *reinterpret_cast<bf16x8*>(k_phi + kphi_offset<D>((size_t)bh * Tn + j, mt0 + a, ks, lane)) = kf[a];
      }
#pragma unroll
      for (int b = 0; b < HS::kNtw; b++) {
        bf16x8 vf = v_fragment<PaddedLayout<D>>(vtile, ks, 32 * (nt0 + b), lane);
#pragma unroll
        for (int a = 0; a < HS::kMtw; a++) hacc[a][b] = mfma_bf16(kf[a], vf, hacc[a][b]);
      }
    }
#pragma unroll
    for (int a = 0; a < HS::kMtw; a++) {
      const float z = half_sum(zsum[a]);
      zacc[a] += z;
      if (g == 0 && nt0 == 0) z_blocks[((size_t)bh * Tn + j) * D + 32 * (mt0 + a) + lane] = z;
    }
  }
  float* ph = partial + (size_t)blockIdx.x * (D * D + D);
#pragma unroll
  for (int a = 0; a < HS::kMtw; a++) {
#pragma unroll
    for (int b = 0; b < HS::kNtw; b++)
#pragma unroll
      for (int e = 0; e < 16; e++) {
        const int c = 32 * (mt0 + a) + 8 * (e / 4) + 4 * g + e % 4;
        ph[c * D + 32 * (nt0 + b) + lane % 32] = hacc[a][b][e];
      }
    if (g == 0 && nt0 == 0) ph[D * D + 32 * (mt0 + a) + lane] = zacc[a];
  }
}

hipError_t launch_kv_state_bf16(const Shape& s, const uint16_t* k, const uint16_t* v, const double* k_mean,
                                float* k_stats, float* partial, uint16_t* k_phi, float* z_blocks, uint8_t* k_codes,
                                float* k_scale, uint8_t* v_codes, float* v_scale, hipStream_t stream) {
  dim3 grid((unsigned)(s.BH * s.chunks));
#define SLA2_KV(DD, QQ)                                                                                          \
  kv_state_bf16_kernel<DD, QQ><<<grid, 256, 0, stream>>>(k, v, k_mean, k_stats, partial, k_phi, z_blocks, k_codes, \
                                                         k_scale, v_codes, v_scale, s.sin, s.H, s.N, s.Tn, s.chunks, \
                                                         s.blocks_per_chunk)
#define SLA2_KV_D(DD)                                                                                  \
  do {                                                                                                 \
    if (s.quant == 3) SLA2_KV(DD, 3); else if (s.quant == 2) SLA2_KV(DD, 2);                           \
    else if (s.quant == 1) SLA2_KV(DD, 1); else SLA2_KV(DD, 0);                                        \
  } while (0)
  if (s.d == 128) SLA2_KV_D(128);
  else SLA2_KV_D(64);
#undef SLA2_KV_D
#undef SLA2_KV
  return hipGetLastError();
}

// =============================================================================================
// attn_mfma
// =============================================================================================
enum AttnMode { kSparseBf16 = 0, kSparseFp8 = 1, kDenseBf16 = 2, kSparseInt8 = 3, kSparseFp8V = 4 };


// LDS carve-up.  Loop: two buffers, each one K tile (bf16, or 8-bit codes), one V tile (bf16) and, when
// V is quantised for the second product, one tile of its codes,
// all in the swizzled layout the load unit fills directly.  Epilogue: H_i^T as bf16 [D][D+8] and the
// output tile [BQ][D+8], overlaying the tile buffers.
template <int D, int BQ, bool FP8, bool VQ = false> struct AttnSmem {
  static constexpr int kLd = TileGeom<D>::kLd;
  static constexpr int kVBytes = SwizzledLayout<D>::kTileBytes;
  static constexpr int kKBytes = FP8 ? SwizzledLayout8<D>::kTileBytes : kVBytes;
  static constexpr int kVqBytes = VQ ? SwizzledLayoutVq<D>::kTileBytes : 0;   // e4m3 codes of V, when P V is an FP8 product
  static constexpr int kBufBytes = kKBytes + kVBytes + kVqBytes;
  static constexpr int kLoopBytes = 2 * kBufBytes;
  static constexpr int kEpiBytes = (D + BQ) * kLd * 2;
  static constexpr int kTiles = kLoopBytes > kEpiBytes ? kLoopBytes : kEpiBytes;
  static constexpr int kZsOff = kTiles;                             // float [D]: Z_i
  static constexpr int kRedOff = kZsOff + D * 4;                    // float [4]: block-wide max
  static constexpr int kBytes = kRedOff + 16;
};


// Waves per SIMD the register budget is set for (second launch bound): 2; 1 for d = 128 with 64-row blocks, whose
// two waves hold half of the d x d state each; 3 for d = 64 with 128-row blocks, where the accumulators are small
// enough for 168 registers (measured on a 32,760-token d = 64 input: 6 % faster in FP8 mode, 10 % in bf16 mode;
// with 64-row blocks three waves gain nothing).
template <int D, int BQ, int MODE>
__global__ __launch_bounds__(BQ * 2, (D == 128 && BQ == 64) ? 1 : (D == 64 && BQ == 128) ? 3 : 2) void attn_mfma_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const double* __restrict__ k_mean, const uint16_t* __restrict__ k_phi, const float* __restrict__ z_blocks,
    const uint8_t* __restrict__ k_codes, const float* __restrict__ k_scale, const uint8_t* __restrict__ v_codes,
    const float* __restrict__ v_scale, const float* __restrict__ h_total,
    const float* __restrict__ z_total, const int32_t* __restrict__ block_idx, const float* __restrict__ alpha,
    uint16_t* __restrict__ out, float* __restrict__ lse, uint16_t* __restrict__ o_s_save,
    uint16_t* __restrict__ o_l_save, float* __restrict__ lse_save, uint16_t* __restrict__ h_save,
    float* __restrict__ z_save, Strides sin, Strides sout, int H, int N, int Tm,
    int Tn, int ksel, int alpha_per_block) {
  // FP8 below means "8-bit codes of Q and K": everything the two low-bit modes share.  INT8 marks the
  // places where the integer mode differs (the quantiser of Q and the Q K^T product).
  // FP8V: V is quantised too and P V runs as an FP8 product (the linear branch still reads the bf16 V).
  constexpr bool DENSE = MODE == kDenseBf16, INT8 = MODE == kSparseInt8, FP8V = MODE == kSparseFp8V;
  constexpr bool FP8 = MODE == kSparseFp8 || INT8 || FP8V;
  constexpr int NW = BQ / 32, NT = NW * kWave;
  constexpr int LD = TileGeom<D>::kLd;
  constexpr int KS = D / 16;            // contraction steps over the head dimension
  constexpr int ET = D / 32;            // 32-wide tiles over the head dimension
  typedef HSplit<D, NW> HS;
  typedef AttnSmem<D, BQ, FP8, FP8V> SM;
  typedef SwizzledLayout<D> SL;
  typedef SwizzledLayout8<D> SL8;
  // Loads and LDS reads of the main loop are issued untracked and waited for by count (see
  // load_untracked).  The one exception is the shape with the highest register pressure, bf16
  // operands at d = 128 with two workgroups per CU: holding reads in flight costs registers it
  // does not have, and the compiler-tracked form is the faster one there.
  constexpr bool kManual = FP8;
  // global -> LDS transfers one wave issues per tile (1 KB each): V, and K in bf16 or e4m3
  constexpr int kDmaOps = kTileTokens * D * 2 / 1024 / NW + kTileTokens * D * (FP8 ? 1 : 2) / 1024 / NW +
                          (FP8V ? kTileTokens * D / 1024 / NW : 0);
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  float* zs = reinterpret_cast<float*>(smem + SM::kZsOff);
  float* red = reinterpret_cast<float*>(smem + SM::kRedOff);
  auto kbuf = [&](int buf) { return smem + buf * SM::kBufBytes; };
  auto vbuf = [&](int buf) { return reinterpret_cast<uint16_t*>(smem + buf * SM::kBufBytes + SM::kKBytes); };
  auto vqbuf = [&](int buf) { return smem + buf * SM::kBufBytes + SM::kKBytes + SM::kVBytes; };

  // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  Consecutive query blocks of
  // a head share key/value tiles: every head is cut into 8 runs of consecutive blocks, one per XCD, and
  // all XCDs work through the heads in the same order - the tiles in flight then belong to one or two
  // heads, which the memory-side cache holds whole.
  const int per_head = (Tm + kXcds - 1) / kXcds;
  const int bh = (blockIdx.x / kXcds) / per_head, i = (blockIdx.x % kXcds) * per_head + (blockIdx.x / kXcds) % per_head;
  if (i >= Tm) return;
  const int h = bh % H;
  const int tid = threadIdx.x, lane = tid % kWave, g = lane / 32;
  const int w = __builtin_amdgcn_readfirstlane(tid / kWave);   // wave index, known to be uniform
  const int row0 = i * BQ;
  const int rows_valid = min(BQ, N - row0);
  const uint16_t* qh = q + head_offset(sin, bh, H);
  const uint16_t* kh = k + head_offset(sin, bh, H);
  const uint16_t* vh = v + head_offset(sin, bh, H);
  const int tok_stride = sin.n;                      // elements between consecutive tokens of q, k, v
  const int32_t* sel = DENSE ? nullptr : block_idx + ((size_t)bh * Tm + i) * ksel;
  const int ntiles = DENSE ? Tn : ksel;
  const int mt0 = HS::mt0(w), nt0 = HS::nt0(w);
  const size_t blk0 = (size_t)bh * Tn;   // first key block of this head in the per-block arrays
  // Key block of tile s.  The indices (and the FP8 scales) are fetched one and two tiles ahead of
  // their use: a scalar load consumed right away stalls the wave for its whole latency.
  auto tile_block = [&](int s) { return DENSE ? min(s, Tn - 1) : sel[min(s, ntiles - 1)]; };
  int j_cur = ntiles > 0 ? tile_block(0) : 0, j_nxt = ntiles > 0 ? tile_block(1) : 0;
  float sk_cur = 1.f;
  if constexpr (FP8) sk_cur = k_scale[blk0 + j_cur];
  // FP8V: O^T is carried in units of the V scale of the tile being added (the factor between two tiles
  // joins the online-softmax correction); sv_cur is the scale of the coming tile, sv_prev of the last one
  float sv_cur = 1.f, sv_prev = 1.f;
  if constexpr (FP8V) sv_cur = sv_prev = ntiles > 0 ? v_scale[blk0 + j_cur] : 1.f;

  // tile s: global memory -> LDS buffer `buf`, no registers involved (completion: vmcnt)
  auto dma = [&](int j, int buf) {
    const int t0 = j * kTileTokens, valid = min(kTileTokens, N - t0);
    if constexpr (FP8) dma_tile8<D, NW>(k_codes + (blk0 + j) * kTileTokens * D, kbuf(buf), w, lane);
    else if (kManual && valid == kTileTokens) dma_tile_full<D, NW>(kh + (size_t)t0 * tok_stride, tok_stride, reinterpret_cast<uint16_t*>(kbuf(buf)), w, lane);
    else dma_tile<D, NW>(kh + (size_t)t0 * tok_stride, tok_stride, valid, reinterpret_cast<uint16_t*>(kbuf(buf)), w, lane);
    if (kManual && valid == kTileTokens) dma_tile_full<D, NW>(vh + (size_t)t0 * tok_stride, tok_stride, vbuf(buf), w, lane);
    else dma_tile<D, NW>(vh + (size_t)t0 * tok_stride, tok_stride, valid, vbuf(buf), w, lane);
    if constexpr (FP8V) dma_tile_vq<D, NW>(v_codes + (blk0 + j) * kTileTokens * D, vqbuf(buf), w, lane);
  };

  if (ntiles > 0) dma(j_cur, 0);

  // Q fragments (B operand of S^T = K Q^T): lane <- Q[row0 + 32 w + l%32][16 ks + 8 g + 0..7]
  bf16x8 qf[KS];
  {
    const int r = min(32 * w + lane % 32, rows_valid - 1);   // rows past the end repeat the last one; never stored
    const uint16_t* src = qh + (size_t)(row0 + r) * tok_stride;
    // bf16 product: fragment ks = columns 16 ks + 8 g + 0..7.  FP8 product (64 deep): the lane's
    // operand of step ks2 is columns 64 ks2 + 32 g + 0..31, held as fragments 4 ks2 + 0..3.
    // INT8 product (32 deep): columns 32 ks4 + 16 g + 0..15, fragments 2 ks4 + 0..1.
#pragma unroll
    for (int ks = 0; ks < KS; ks++)
      qf[ks] = *reinterpret_cast<const bf16x8*>(
          src + (INT8 ? 32 * (ks / 2) + 16 * g + 8 * (ks % 2) : FP8 ? 64 * (ks / 4) + 32 * g + 8 * (ks % 4) : 16 * ks + 8 * g));
  }
  // The state accumulators start at -H_total (and -Z_total): the loop adds the h_j and z_j of the selected
  // blocks, which leaves -(H_total - sum) = -H_i.  The d x d total is read here, behind the first tile's
  // transfer, instead of in the epilogue, where a wave would wait for it with nothing else to do.
  f32x16 hacc[HS::kMtw][HS::kNtw];
  float zsel[HS::kMtw];
#pragma unroll
  for (int a = 0; a < HS::kMtw; a++) {
    zsel[a] = 0.f;
#pragma unroll
    for (int b = 0; b < HS::kNtw; b++)
#pragma unroll
      for (int e = 0; e < 16; e++) hacc[a][b][e] = 0.f;
  }
  if constexpr (!DENSE) {
    const float* htot = h_total + (size_t)bh * D * D;
#pragma unroll
    for (int a = 0; a < HS::kMtw; a++) {
#pragma unroll
      for (int b = 0; b < HS::kNtw; b++)
#pragma unroll
        for (int e = 0; e < 16; e++)
          hacc[a][b][e] = -htot[(32 * (mt0 + a) + 8 * (e / 4) + 4 * g + e % 4) * D + 32 * (nt0 + b) + lane % 32];
      zsel[a] = -z_total[(size_t)bh * D + 32 * (mt0 + a) + lane % 32];
    }
  }
  // Everything issued so far is settled here, on every path into the main loop; a pending load
  // left over from the prologue would otherwise put a vmcnt wait in front of every use of a Q
  // fragment inside the loop and drain the tile prefetch with it.
  __builtin_amdgcn_s_waitcnt(kVmcnt0);
  // FP8: quant(Q_i) with one scale for the whole query block (Sec. 5)
  long qf8[FP8 ? KS : 1];
  float s_q = 1.f;
  if constexpr (FP8) {
    float amax = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ks++)
#pragma unroll
      for (int e = 0; e < 8; e++) amax = fmaxf(amax, fabsf((float)qf[ks][e]));
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) amax = fmaxf(amax, __shfl_xor(amax, o));
    if (lane == 0) red[w] = amax;
    __syncthreads();
    amax = red[0];
#pragma unroll
    for (int x = 1; x < NW; x++) amax = fmaxf(amax, red[x]);
    constexpr float kCodeMax = INT8 ? kInt8Max : kE4M3Max;
    const float inv = amax > 0.f ? kCodeMax / amax : 1.f;
    s_q = amax > 0.f ? amax / kCodeMax : 1.f;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      float y[8];
#pragma unroll
      for (int e = 0; e < 8; e++) y[e] = fminf(fmaxf((float)qf[ks][e] * inv, -kCodeMax), kCodeMax);
      int lo = 0, hi = 0;
      if constexpr (INT8) {
        lo = pack_int8(y[0], y[1], y[2], y[3]);
        hi = pack_int8(y[4], y[5], y[6], y[7]);
      } else {
        lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], lo, false);
        lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], lo, true);
        hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[4], y[5], hi, false);
        hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[6], y[7], hi, true);
      }
      qf8[ks] = (long)(((unsigned long)(unsigned)hi << 32) | (unsigned)lo);
    }
  }
  __syncthreads();                                   // tile 0 is in LDS for everyone

  f32x16 oacc[ET];
#pragma unroll
  for (int et = 0; et < ET; et++)
#pragma unroll
    for (int e = 0; e < 16; e++) oacc[et][e] = 0.f;
  // running max and sum of this lane's query row, in the log2 domain.  In FP8 mode P is carried
  // scaled by 2^8 (the rounding grid of P, see sla2.h): the factor cancels in O / l.
  float m_run = -INFINITY, l_run = 0.f;
  constexpr float kPShift = FP8 ? 8.f : 0.f;
  const float c0 = kLog2e * rsqrtf((float)D);        // scores are used as S * log2(e) / sqrt(d)

  for (int s = 0; s < ntiles; s++) {
    const int buf = s & 1;
    const int j = j_cur;
    const int valid = min(kTileTokens, N - j * kTileTokens);
    const float sk = sk_cur;
    const int j_nn = tile_block(s + 2);                // consumed in the next iteration
    if constexpr (FP8) sk_cur = k_scale[blk0 + j_nxt];
    const float sv = sv_cur;
    if constexpr (FP8V) sv_cur = v_scale[blk0 + j_nxt];
    // K^phi fragments and z_j of this tile straight from global memory into registers (no other
    // wave needs them); they are consumed after the softmax.  They are issued before the next
    // tile's transfer and, since vmcnt retires in order, are complete once at most kDmaOps
    // operations are outstanding.  The loads are opaque to the compiler on purpose: its own
    // bookkeeping across the conditional transfer below falls back to vmcnt(0) at their first
    // use, which stalls every iteration on the tile that was just requested.
    bf16x8 kphi[DENSE ? 1 : HS::kMtw][kTileTokens / 16];
    float zj[DENSE ? 1 : HS::kMtw];
    auto state_loads = [&]() {
      if constexpr (!DENSE) {
#pragma unroll
        for (int a = 0; a < HS::kMtw; a++) {
#pragma unroll
          for (int ks = 0; ks < kTileTokens / 16; ks++)
            kphi[a][ks] = load_maybe_tracked<bf16x8, kManual>(k_phi + kphi_offset<D>(blk0 + j, mt0 + a, ks, lane));
          zj[a] = load_maybe_tracked<float, kManual>(z_blocks + (blk0 + j) * D + 32 * (mt0 + a) + lane % 32);
          if constexpr (!kManual) zsel[a] += zj[a];
        }
      }
    };
    auto next_tile = [&]() {
      if (s + 1 < ntiles) dma(j_nxt, buf ^ 1);       // next tile -> other buffer
    };
    // With the reads under this kernel's own control (low-bit modes) the requests for the rest of the
    // tile's data are placed inside the score product: the fragment loads behind its operand reads, the
    // next tile's transfer behind its matrix instructions - some hundred instructions that otherwise
    // stand in front of it, on a wave whose progress is bound by its own chain of dependent steps.
    constexpr bool kRequestsInsideScores = kManual;
    if constexpr (!kRequestsInsideScores) {
      state_loads();
      next_tile();
    }
    const uint16_t* vt = vbuf(buf);
    // Two waves share a SIMD.  The one that is issuing matrix products is given the higher issue priority, so
    // that the matrix pipe is fed while the other wave's softmax fills the gaps (measured: 2 % on the
    // sparse modes; the dense comparator, all of whose waves are in step, loses with it).
    if constexpr (!DENSE) __builtin_amdgcn_s_setprio(2);
    // ---- S^T = K Q^T (keys x query rows), two 32-key halves ----
    f32x16 sacc[2];
#pragma unroll
    for (int mt = 0; mt < 2; mt++)
#pragma unroll
      for (int e = 0; e < 16; e++) sacc[mt][e] = 0.f;
    if constexpr (INT8) {
      // 32-deep integer products (v_mfma_i32_32x32x32_i8: lane l holds row l % 32, contraction indices
      // 16 (l / 32) + 0..15): the operand of (step ks4, key half mt) is 16 consecutive codes of key row
      // 32 mt + l % 32 - one 16-byte read at (address of step 0) ^ 32 ks4 in the pair-swizzled tile.
      // Sums of 128 products of codes stay below 2^21: exact in the int32 accumulator and in fp32.
      constexpr int KS4 = D / 32;
      const unsigned ka = lds_address(kbuf(buf) + SL8::offset(lane % 32, 16 * g));
      u32x4 kq[KS4][2];
#pragma unroll
      for (int ks4 = 0; ks4 < KS4; ks4++) {
        kq[ks4][0] = lds_read16_untracked<0>(ka ^ (32u * ks4));
        kq[ks4][1] = lds_read16_untracked<32 * D>(ka ^ (32u * ks4));
      }
      if constexpr (kRequestsInsideScores) state_loads();
      i32x16 iacc[2];
#pragma unroll
      for (int mt = 0; mt < 2; mt++)
#pragma unroll
        for (int e = 0; e < 16; e++) iacc[mt][e] = 0;
#pragma unroll
      for (int ks4 = 0; ks4 < KS4; ks4++)
#pragma unroll
        for (int mt = 0; mt < 2; mt++) {
          wait_lgkmcnt(2 * (KS4 - 1 - ks4) + 1 - mt);
          settle(kq[ks4][mt]);
          const u32x4 kk = kq[ks4][mt];
          const i32x4 a = {(int)kk[0], (int)kk[1], (int)kk[2], (int)kk[3]};
          const i32x4 b = {(int)(unsigned)((unsigned long)qf8[2 * ks4]), (int)(unsigned)((unsigned long)qf8[2 * ks4] >> 32),
                           (int)(unsigned)((unsigned long)qf8[2 * ks4 + 1]), (int)(unsigned)((unsigned long)qf8[2 * ks4 + 1] >> 32)};
          iacc[mt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, iacc[mt], 0, 0, 0);
        }
      if constexpr (kRequestsInsideScores) next_tile();
#pragma unroll
      for (int mt = 0; mt < 2; mt++)
#pragma unroll
        for (int e = 0; e < 16; e++) sacc[mt][e] = (float)iacc[mt][e];
    } else if constexpr (FP8) {
      // 64-deep products: the operand of (step ks2, key half mt) is 32 consecutive codes of key row
      // 32 mt + l % 32, two 16-byte reads.  The swizzle is an XOR on the pair bits of the address,
      // so step ks2 sits at (address of step 0) ^ 64 ks2; all reads of a tile are issued up front.
      static_assert(D % 64 == 0, "the FP8 product consumes the head dimension 64 at a time");
      constexpr int KS2 = D / 64;
      const unsigned ka = lds_address(kbuf(buf) + SL8::offset(lane % 32, 32 * g));
      u32x4 klo[KS2][2], khi[KS2][2];
#pragma unroll
      for (int ks2 = 0; ks2 < KS2; ks2++) {
        klo[ks2][0] = lds_read16_untracked<0>(ka ^ (64u * ks2));
        khi[ks2][0] = lds_read16_untracked<16>(ka ^ (64u * ks2));
        klo[ks2][1] = lds_read16_untracked<32 * D>(ka ^ (64u * ks2));
        khi[ks2][1] = lds_read16_untracked<32 * D + 16>(ka ^ (64u * ks2));
      }
      if constexpr (kRequestsInsideScores) state_loads();
#pragma unroll
      for (int ks2 = 0; ks2 < KS2; ks2++)
#pragma unroll
        for (int mt = 0; mt < 2; mt++) {
          wait_lgkmcnt(2 * (2 * (KS2 - 1 - ks2) + 1 - mt));
          settle(klo[ks2][mt]);
          settle(khi[ks2][mt]);
          const u32x4 lo = klo[ks2][mt], hi = khi[ks2][mt];
          const i32x8 a = {(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
          i32x8 b;
#pragma unroll
          for (int x = 0; x < 4; x++) {
            b[2 * x] = (int)(unsigned)((unsigned long)qf8[4 * ks2 + x]);
            b[2 * x + 1] = (int)(unsigned)((unsigned long)qf8[4 * ks2 + x] >> 32);
          }
          sacc[mt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, sacc[mt], 0, 0, 0, 0, 0, 0);   // e4m3 x e4m3, no scales
        }
      if constexpr (kRequestsInsideScores) next_tile();
    } else {
      const uint16_t* kt = reinterpret_cast<const uint16_t*>(kbuf(buf));
#pragma unroll
      for (int ks = 0; ks < KS; ks++)
#pragma unroll
        for (int mt = 0; mt < 2; mt++)
          sacc[mt] = mfma_bf16(row_fragment<SL>(kt, 32 * mt + lane % 32, 16 * ks + 8 * g), qf[ks], sacc[mt]);
    }
    j_cur = j_nxt;
    j_nxt = j_nn;
    if constexpr (!DENSE) __builtin_amdgcn_s_setprio(0);   // softmax: the other wave's matrix products go first
    // ---- online softmax of this lane's query row over the 64 keys ----
    const float c1 = FP8 ? c0 * s_q * sk : c0;       // dequantisation folded into the score scale
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
    mx = half_max(mx) * c1;
    // The reference of the exponentials.  With P rounded to a grid (low-bit modes) it is the running maximum,
    // as Alg. 2 states it.  Otherwise any reference gives the same O / l, and the one in use is kept while the
    // maximum of the row stays within 2^kLazy of it: O^T, l then need no rescaling in most tiles (the weights
    // reach at most 2^kLazy, harmless in bf16 and fp32).  The decision is taken for the whole wave.
    constexpr float kLazy = 8.f;
    bool rescale = true;
    if constexpr (!FP8) rescale = __builtin_amdgcn_ballot_w64(mx > m_run + kLazy) != 0;   // first tile: m_run = -inf
    const float m_new = rescale ? fmaxf(m_run, mx) : m_run;   // finite: a tile holds at least one key
    const float m_off = m_new - kPShift;
    float rs = 0.f;
    bf16x8 pf[FP8V ? 1 : 4];                         // P^T fragments, token order
    i32x8 pb;                                        // FP8V: the e4m3 codes of P^T, byte 16 mt + e of the lane's half
    int codes = 0;
#pragma unroll
    for (int mt = 0; mt < 2; mt++)
#pragma unroll
      for (int e = 0; e < 16; e += 2) {
        const float p0 = fast_exp2(sacc[mt][e] * c1 - m_off);
        const float p1 = fast_exp2(sacc[mt][e + 1] * c1 - m_off);
        rs += p0 + p1;                               // the denominator keeps the un-rounded P
        if constexpr (FP8V) {
          const int q = 4 * mt + e / 4;              // two codes into the lower or upper half of dword q
          if (e % 4 == 0) pb[q] = __builtin_amdgcn_cvt_pk_fp8_f32(p0, p1, 0, false);
          else pb[q] = __builtin_amdgcn_cvt_pk_fp8_f32(p0, p1, pb[q], true);
        } else if constexpr (FP8) {
          // quant(P): e4m3 grid.  The instruction keeps the other half of its destination; feeding it the
          // previous pair's register (dead by now) instead of a zero saves a register move per pair
          codes = __builtin_amdgcn_cvt_pk_fp8_f32(p0, p1, codes, false);
          typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
          const bf16x2 pq = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(codes, 1.0f, false);
          pf[2 * mt + e / 8][e % 8] = pq[0];
          pf[2 * mt + e / 8][e % 8 + 1] = pq[1];
        } else {
          pf[2 * mt + e / 8][e % 8] = (__bf16)p0;
          pf[2 * mt + e / 8][e % 8 + 1] = (__bf16)p1;
        }
      }
    rs = half_sum(rs);
    if (rescale) {
      const float corr = fast_exp2(m_run - m_new);   // 0 on the first tile
      l_run *= corr;
      m_run = m_new;
      const float corr_o = FP8V ? corr * (sv_prev / sv) : corr;   // FP8V: also from the last tile's V scale to this one's
      sv_prev = sv;
#pragma unroll
      for (int et = 0; et < ET; et++)
#pragma unroll
        for (int e = 0; e < 16; e++) oacc[et][e] *= corr_o;
    }
    l_run += rs;

    if constexpr (!DENSE) __builtin_amdgcn_s_setprio(2);   // matrix products again
    if constexpr (!DENSE) {
      if constexpr (kManual) {
        // the register loads issued at the top have landed; the tile transfer may still be in flight
        if (s + 1 < ntiles) wait_vmcnt<kDmaOps>();
        else wait_vmcnt<0>();
#pragma unroll
        for (int a = 0; a < HS::kMtw; a++) {
#pragma unroll
          for (int ks = 0; ks < kTileTokens / 16; ks++) settle(kphi[a][ks]);
          settle(zj[a]);
        }
#pragma unroll
        for (int a = 0; a < HS::kMtw; a++) zsel[a] += zj[a];
      }
    }
    if constexpr (FP8V) {
      // O^T += Vhat^T Ptilde^T as 64-deep FP8 products, one per 32-channel tile: the operand is the half
      // row (l / 32) of channel row 32 et + l % 32 of the code tile, two 16-byte reads
      typedef SwizzledLayoutVq<D> SLV;
      const unsigned qa = lds_address(vqbuf(buf) + SLV::offset(lane % 32, 2 * g));
      u32x4 vq_lo[ET], vq_hi[ET];
#pragma unroll
      for (int et = 0; et < ET; et++) {
        vq_lo[et] = lds_read16_untracked_at<32 * kTileTokens>(qa, et);
        vq_hi[et] = lds_read16_untracked_at<32 * kTileTokens>(qa ^ 16u, et);
      }
#pragma unroll
      for (int et = 0; et < ET; et++) {
        wait_lgkmcnt(2 * (ET - 1 - et));
        settle(vq_lo[et]);
        settle(vq_hi[et]);
        const u32x4 lo = vq_lo[et], hi = vq_hi[et];
        const i32x8 a = {(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
        oacc[et] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, pb, oacc[et], 0, 0, 0, 0, 0, 0);
      }
    }
    // ---- O^T += V^T P^T, and the d x d state of this block: h += K^phi^T V ----
    // address of this lane's first transposing read of fragment (ks = 0, et = 0), cf. read_tr4
    const unsigned va = lds_address(vt + SL::offset(4 * g + (lane % 16) / 4, 16 * ((lane / 16) % 2) + 4 * (lane % 4)));
    unsigned vaddr[ET];                              // one address per 32-channel tile; the token step is an immediate
#pragma unroll
    for (int et = 0; et < ET; et++) vaddr[et] = va ^ (64u * et);
    u32x2 vlo[3], vhi[3];
#pragma unroll
    for (int ks = 0; ks < kTileTokens / 16; ks++) {
      if constexpr (!kManual && (HS::kNtw == ET || DENSE)) {   // every V fragment feeds both products
#pragma unroll
        for (int et = 0; et < ET; et++) {
          bf16x8 vf = v_fragment<SL>(vt, ks, 32 * et, lane);
          if constexpr (!FP8V) oacc[et] = mfma_bf16(vf, pf[ks], oacc[et]);
          if constexpr (!DENSE) {
#pragma unroll
            for (int a = 0; a < HS::kMtw; a++) hacc[a][et] = mfma_bf16(kphi[a][ks], vf, hacc[a][et]);
          }
        }
      } else if constexpr (HS::kNtw == ET || DENSE) {       // the same with the reads kept in flight
        // fragment f = ks ET + et: two transposing reads (tokens 16 ks + 4 g.. and + 8), kept kVAhead
        // fragments ahead of the products.  Row swizzle and lane terms are the same for every
        // fragment of a lane, so fragment (ks, et) sits at (va ^ 64 et) + 32 D ks.
        constexpr int kVAhead = FP8 ? 2 : 1, kFrags = (kTileTokens / 16) * ET;
        if (ks == 0) {
#pragma unroll
          for (int f = 0; f < kVAhead; f++) {
            vlo[f] = lds_read_tr_untracked_at<8 * D * 2>(vaddr[f % ET], 2 * (f / ET));
            vhi[f] = lds_read_tr_untracked_at<8 * D * 2>(vaddr[f % ET], 2 * (f / ET) + 1);
          }
        }
#pragma unroll
        for (int et = 0; et < ET; et++) {
          const int f = ks * ET + et;
          if (f + kVAhead < kFrags) {
            const int f2 = f + kVAhead;
            vlo[f2 % (kVAhead + 1)] = lds_read_tr_untracked_at<8 * D * 2>(vaddr[f2 % ET], 2 * (f2 / ET));
            vhi[f2 % (kVAhead + 1)] = lds_read_tr_untracked_at<8 * D * 2>(vaddr[f2 % ET], 2 * (f2 / ET) + 1);
          }
          const int left = kFrags - 1 - f;
          wait_lgkmcnt(2 * (left < kVAhead ? left : kVAhead));
          u32x2& lo = vlo[f % (kVAhead + 1)];
          u32x2& hi = vhi[f % (kVAhead + 1)];
          settle(lo);
          settle(hi);
          const u32x4 v4 = {lo[0], lo[1], hi[0], hi[1]};
          const bf16x8 vf = __builtin_bit_cast(bf16x8, v4);
          if constexpr (!FP8V) oacc[et] = mfma_bf16(vf, pf[ks], oacc[et]);
          if constexpr (!DENSE) {
#pragma unroll
            for (int a = 0; a < HS::kMtw; a++) hacc[a][et] = mfma_bf16(kphi[a][ks], vf, hacc[a][et]);
          }
        }
      } else {
#pragma unroll
        for (int et = 0; et < ET; et++) {
          bf16x8 vf = v_fragment<SL>(vt, ks, 32 * et, lane);
          if constexpr (!FP8V) oacc[et] = mfma_bf16(vf, pf[ks], oacc[et]);
        }
#pragma unroll
        for (int b = 0; b < HS::kNtw; b++) {
          bf16x8 vf = v_fragment<SL>(vt, ks, 32 * (nt0 + b), lane);
#pragma unroll
          for (int a = 0; a < HS::kMtw; a++) hacc[a][b] = mfma_bf16(kphi[a][ks], vf, hacc[a][b]);
        }
      }
    }
    __builtin_amdgcn_s_waitcnt(kVmcnt0);             // the next tile has landed in LDS ...
    __syncthreads();                                 // ... for everyone, and this tile's buffer is free
  }

  if constexpr (!DENSE) __builtin_amdgcn_s_setprio(0);
  // ================= epilogue =================
  const float inv_l = l_run > 0.f ? 1.f / l_run : 0.f;
  const int qrow = 32 * w + lane % 32;               // this lane's query row inside the block
  if (lse != nullptr || lse_save != nullptr) {
    // Alg. 2 defines L on the smoothed keys.  The bf16 products above use the raw K, whose scores
    // are larger by q . colmean(K) / sqrt(d) in every column of a row (the softmax cancels it);
    // the FP8 codes are those of the smoothed K already.
    float qmu = 0.f;
    if (!DENSE && !FP8) {
#pragma unroll
      for (int ks = 0; ks < KS; ks++)
#pragma unroll
        for (int e = 0; e < 8; e++) qmu += (float)qf[ks][e] * (float)k_mean[(size_t)bh * D + 16 * ks + 8 * g + e];
      qmu = half_sum(qmu);
    }
    if (g == 0 && qrow < rows_valid) {
      const float L =
          l_run > 0.f ? (m_run - kPShift + __log2f(l_run)) * 0.6931471805599453f - qmu * rsqrtf((float)D) : -INFINITY;
      if (lse != nullptr) lse[(size_t)bh * N + row0 + qrow] = L;
      if (lse_save != nullptr) lse_save[(size_t)bh * N + row0 + qrow] = L;
    }
  }

  if constexpr (FP8) {
    // the bf16 Q fragments were dropped after quantisation to keep two waves per SIMD; the linear
    // branch needs them once more
    const int r = min(32 * w + lane % 32, rows_valid - 1);
    const uint16_t* src = qh + (size_t)(row0 + r) * tok_stride + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) qf[ks] = *reinterpret_cast<const bf16x8*>(src + 16 * ks);
  }
  uint16_t* ht = reinterpret_cast<uint16_t*>(smem);  // H_i^T as bf16 [e][c], row stride LD
  uint16_t* os = ht + D * LD;                        // output tile [BQ][LD]
  f32x16 lacc[ET];
  float inv_den = 0.f;
  if constexpr (!DENSE) {
    // H_i^T = -(accumulated)^T as bf16, Z_i likewise
#pragma unroll
    for (int a = 0; a < HS::kMtw; a++) {
#pragma unroll
      for (int b = 0; b < HS::kNtw; b++) {
        const int e_col = 32 * (nt0 + b) + lane % 32;
#pragma unroll
        for (int v4 = 0; v4 < 4; v4++) {
          const int cc = 32 * (mt0 + a) + 8 * v4 + 4 * g;
          bf16x4 pk;
#pragma unroll
          for (int r = 0; r < 4; r++) pk[r] = (__bf16)(-hacc[a][b][4 * v4 + r]);
          *reinterpret_cast<bf16x4*>(ht + e_col * LD + cc) = pk;
        }
      }
      // zsel holds the same sum on both lane halves (each half added z_j of channel l % 32)
      if (g == 0 && nt0 == 0) zs[32 * (mt0 + a) + lane] = -zsel[a];
    }
    // Q^phi = softmax_d(Q) of this lane's row, kept as fragments - without its normaliser, which cancels
    // between Q^phi H_i and Q^phi Z_i
    float qx[KS][8];
    float qm = -INFINITY;
#pragma unroll
    for (int ks = 0; ks < KS; ks++)
#pragma unroll
      for (int e = 0; e < 8; e++) {
        qx[ks][e] = (float)qf[ks][e];
        qm = fmaxf(qm, qx[ks][e]);
      }
    qm = half_max(qm);
#pragma unroll
    for (int ks = 0; ks < KS; ks++)
#pragma unroll
      for (int e = 0; e < 8; e++) qx[ks][e] = fast_exp2((qx[ks][e] - qm) * kLog2e);
    __syncthreads();                                 // H_i^T and Z_i visible
    float den = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      const f32x4 z0 = *reinterpret_cast<const f32x4*>(zs + 16 * ks + 8 * g);
      const f32x4 z1 = *reinterpret_cast<const f32x4*>(zs + 16 * ks + 8 * g + 4);
#pragma unroll
      for (int e = 0; e < 8; e++) {
        den += qx[ks][e] * (e < 4 ? z0[e] : z1[e - 4]);
        qf[ks][e] = (__bf16)qx[ks][e];
      }
    }
    den = half_sum(den);
    inv_den = ksel >= Tn ? 0.f : 1.f / den;          // every block selected: nothing left for the linear branch
    // O_l^T = H_i^T Q^phi^T (the four accumulators take turns, so that no product waits for the one before it)
#pragma unroll
    for (int et = 0; et < ET; et++)
#pragma unroll
      for (int e = 0; e < 16; e++) lacc[et][e] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ks++)
#pragma unroll
      for (int et = 0; et < ET; et++) {
        bf16x8 a = *reinterpret_cast<const bf16x8*>(ht + (32 * et + lane % 32) * LD + 16 * ks + 8 * g);
        lacc[et] = mfma_bf16(a, qf[ks], lacc[et]);
      }
  }
  // ---- mix (Eq. 13), transpose through LDS, coalesced store ----
  const float al = DENSE ? 1.f : alpha[alpha_per_block ? (size_t)h * Tm + i : (size_t)h];
  const float ws = al * inv_l * (FP8V ? sv_prev : 1.f), wl = (1.f - al) * inv_den;   // FP8V: back from the last tile's V scale
#pragma unroll
  for (int et = 0; et < ET; et++)
#pragma unroll
    for (int v4 = 0; v4 < 4; v4++) {
      bf16x4 pk;
#pragma unroll
      for (int r = 0; r < 4; r++) {
        float o = ws * oacc[et][4 * v4 + r];
        if constexpr (!DENSE) o += wl * lacc[et][4 * v4 + r];
        pk[r] = (__bf16)o;
      }
      *reinterpret_cast<bf16x4*>(os + qrow * LD + 32 * et + 8 * v4 + 4 * g) = pk;
    }
  __syncthreads();
  uint16_t* oh = out + head_offset(sout, bh, H) + (size_t)row0 * sout.n;
  for (int idx = tid; idx < BQ * (D / 8); idx += NT) {
    const int r = idx / (D / 8), ch = idx % (D / 8);
    if (r < rows_valid) *reinterpret_cast<u32x4*>(oh + (size_t)r * sout.n + 8 * ch) = *reinterpret_cast<const u32x4*>(os + r * LD + 8 * ch);
  }
  if constexpr (!DENSE) {
    if (h_save != nullptr) {
      // H_i^T (bf16 [e][c], as the product above consumed it) and Z_i, kept for the backward pass
      uint16_t* dst = h_save + ((size_t)bh * Tm + i) * D * D;
      for (int idx = tid; idx < D * (D / 8); idx += NT) {
        const int e = idx / (D / 8), ch = idx % (D / 8);
        *reinterpret_cast<u32x4*>(dst + e * D + 8 * ch) = *reinterpret_cast<const u32x4*>(ht + e * LD + 8 * ch);
      }
      if (tid < D) z_save[((size_t)bh * Tm + i) * D + tid] = zs[tid];
    }
  }
  if (o_s_save != nullptr) {
    // O^s (and O^l, if asked for) on its own ([BH, N, d] contiguous), kept for the backward pass: same
    // route through the transposing tile as the mixed output
    for (int which = 0; which < (o_l_save != nullptr ? 2 : 1); which++) {
      __syncthreads();                                 // the tile has been read out
#pragma unroll
      for (int et = 0; et < ET; et++)
#pragma unroll
        for (int v4 = 0; v4 < 4; v4++) {
          bf16x4 pk;
#pragma unroll
          for (int r = 0; r < 4; r++) {
            float o = which == 0 ? oacc[et][4 * v4 + r] * inv_l * (FP8V ? sv_prev : 1.f) : 0.f;
            if constexpr (!DENSE) {
              if (which == 1) o = lacc[et][4 * v4 + r] * inv_den;
            }
            pk[r] = (__bf16)o;
          }
          *reinterpret_cast<bf16x4*>(os + qrow * LD + 32 * et + 8 * v4 + 4 * g) = pk;
        }
      __syncthreads();
      uint16_t* dst = (which == 0 ? o_s_save : o_l_save) + ((size_t)bh * N + row0) * D;
      for (int idx = tid; idx < BQ * (D / 8); idx += NT) {
        const int r = idx / (D / 8), ch = idx % (D / 8);
        if (r < rows_valid) *reinterpret_cast<u32x4*>(dst + (size_t)r * D + 8 * ch) = *reinterpret_cast<const u32x4*>(os + r * LD + 8 * ch);
      }
    }
  }
}

struct AttnArgs {
  const uint16_t *q, *k, *v;
  const double* k_mean;
  const uint16_t* k_phi;
  const float* z_blocks;
  const uint8_t* k_fp8;
  const float* k_scale;
  const uint8_t* v_codes;
  const float *v_scale, *h_total, *z_total;
  const int32_t* block_idx;
  const float* alpha;
  uint16_t* out;
  float* lse;
  SavedForBackward sv;
};

template <int D, int BQ, int MODE>
static hipError_t launch_attn_t(const Shape& s, const AttnArgs& a, hipStream_t stream) {
  constexpr int smem = AttnSmem<D, BQ, MODE == kSparseFp8 || MODE == kSparseInt8 || MODE == kSparseFp8V, MODE == kSparseFp8V>::kBytes;
  static OncePerDevice once;
  if (hipError_t e = allow_dynamic_lds(once, (const void*)attn_mfma_kernel<D, BQ, MODE>, smem); e != hipSuccess) return e;
  const int Tm = (s.N + BQ - 1) / BQ;
  const int grid = ((Tm + kXcds - 1) / kXcds) * kXcds * s.BH;   // some workgroups of the last run of a head may have no block
  attn_mfma_kernel<D, BQ, MODE><<<dim3((unsigned)grid), BQ * 2, smem, stream>>>(
      a.q, a.k, a.v, a.k_mean, a.k_phi, a.z_blocks, a.k_fp8, a.k_scale, a.v_codes, a.v_scale, a.h_total, a.z_total,
      a.block_idx, a.alpha,
      a.out, a.lse, (uint16_t*)a.sv.o_s, (uint16_t*)a.sv.o_l, a.sv.lse, a.sv.h_i, a.sv.z_i, s.sin, s.sout, s.H, s.N, Tm, s.Tn, s.k,
      s.alpha_per_block ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch_attn_bf16(const Shape& s, const uint16_t* q, const uint16_t* k, const uint16_t* v,
                            const double* k_mean, const uint16_t* k_phi, const float* z_blocks, const uint8_t* k_fp8,
                            const float* k_scale, const uint8_t* v_codes, const float* v_scale,
                            const float* h_total, const float* z_total,
                            const int32_t* block_idx, const float* alpha, uint16_t* out, float* lse,
                            const SavedForBackward& sv, hipStream_t stream) {
  AttnArgs a{q, k, v, k_mean, k_phi, z_blocks, k_fp8, k_scale, v_codes, v_scale, h_total, z_total, block_idx, alpha, out, lse, sv};
#define SLA2_ATTN(DD, QQ)                                                  \
  return s.quant == 3 ? launch_attn_t<DD, QQ, kSparseFp8V>(s, a, stream)   \
       : s.quant == 2 ? launch_attn_t<DD, QQ, kSparseInt8>(s, a, stream)   \
       : s.quant == 1 ? launch_attn_t<DD, QQ, kSparseFp8>(s, a, stream)    \
                      : launch_attn_t<DD, QQ, kSparseBf16>(s, a, stream)
  if (s.d == 128 && s.bq == 128) SLA2_ATTN(128, 128);
  if (s.d == 128 && s.bq == 64) SLA2_ATTN(128, 64);
  if (s.d == 64 && s.bq == 128) SLA2_ATTN(64, 128);
  SLA2_ATTN(64, 64);
#undef SLA2_ATTN
}

hipError_t launch_dense_bf16(const Shape& s, const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* out,
                             hipStream_t stream) {
  AttnArgs a{q, k, v, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, out, nullptr,
             SavedForBackward{nullptr, nullptr, nullptr, nullptr, nullptr}};
  // d = 128: the kernel of its own in sla2_dense.hip (256 query rows per workgroup, the two waves of a SIMD
  // in opposite phases)
  if (s.d == 128) return launch_dense_pp(s, q, k, v, out, stream);
  return launch_attn_t<64, 128, kDenseBf16>(s, a, stream);
}

}  // namespace sla2
