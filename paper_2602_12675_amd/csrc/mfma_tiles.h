// Tile helpers shared by the bf16 / FP8 kernels: LDS staging of 64-token K and V tiles and the
// MFMA operand fragments read from them.  gfx950 only (v_mfma_f32_32x32x16_bf16, ds_read_b64_tr_b16).
//
// Fragment convention of v_mfma_f32_32x32x16_{bf16,fp8}: lane l feeds row (A) / column (B)  l % 32
// with the 8 contraction indices 8 (l / 32) + 0..7; the 32 x 32 fp32 result puts column l % 32,
// rows 8 (v / 4) + 4 (l / 32) + v % 4 (v = 0..15) on lane l.  Because a lane of the result holds
// rows {4g..4g+3, 8+4g..8+4g+3} (g = l / 32) of each 16-row half, a result can be fed back as the
// B operand of the next product without leaving registers if the other operand enumerates the
// contraction index in that same order: "token order" below is
//      token(ks, g, kappa) = 16 ks + 8 (kappa / 4) + 4 g + kappa % 4,   kappa = 0..7.
#pragma once
#include "common.h"

namespace sla2 {

constexpr int kTileTokens = 64;                    // b_kv

template <int D> struct TileGeom {
  static constexpr int kLd = D + 8;                // bf16 elements per LDS row (16-byte padded)
  static constexpr int kTileElems = kTileTokens * kLd;
  static constexpr int kChunksPerRow = D / 8;      // 16-byte chunks per row
};

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// 4 tokens x 16 channels per 16-lane group, transposed on the way out of LDS: on return lane l
// holds tile[row0 + 0..3][col0 + l % 32] (row0 may differ between the two lane halves).
template <int LD>
__device__ __forceinline__ s16x4 read_tr4(const uint16_t* tile, int row0, int col0, int lane) {
  const int row = row0 + (lane % 16) / 4;
  const int col = col0 + 16 * ((lane / 16) % 2) + 4 * (lane % 4);
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(tile + row * LD + col));
}

// V fragment in token order: lane l <- V[token(ks, l/32, 0..7)][col0 + l % 32]   (raw bf16 bits)
template <int LD>
__device__ __forceinline__ bf16x8 v_fragment(const uint16_t* vtile, int ks, int col0, int lane) {
  const int g = lane / 32;
  s16x4 lo = read_tr4<LD>(vtile, 16 * ks + 4 * g, col0, lane);
  s16x4 hi = read_tr4<LD>(vtile, 16 * ks + 8 + 4 * g, col0, lane);
  typedef __attribute__((ext_vector_type(8))) short s16x8;
  s16x8 r = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, r);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// K^phi fragment in token order for channel col0 + l % 32:
//   K^phi[t][c] = exp(k[t][c] - mu[c] - lnZ[t]) = exp2(k log2e - (mu2 + lnz2[t]))
// lnz2: LDS array of 64 floats, lnZ[t] * log2e, +inf for tokens past the end (-> K^phi = 0).
// Adds the 8 fp32 values to zsum (column sums of K^phi, Alg. 2's z).
template <int LD>
__device__ __forceinline__ bf16x8 kphi_fragment(const uint16_t* ktile, const float* lnz2, float mu2, int ks, int col0,
                                                int lane, float& zsum) {
  const int g = lane / 32;
  s16x4 lo = read_tr4<LD>(ktile, 16 * ks + 4 * g, col0, lane);
  s16x4 hi = read_tr4<LD>(ktile, 16 * ks + 8 + 4 * g, col0, lane);
  const f32x4 zl = *reinterpret_cast<const f32x4*>(lnz2 + 16 * ks + 4 * g);
  const f32x4 zh = *reinterpret_cast<const f32x4*>(lnz2 + 16 * ks + 8 + 4 * g);
  bf16x8 r;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    float a = fast_exp2(bf16_bits_to_f32((uint16_t)lo[i]) * kLog2e - (mu2 + zl[i]));
    float b = fast_exp2(bf16_bits_to_f32((uint16_t)hi[i]) * kLog2e - (mu2 + zh[i]));
    zsum += a + b;
    r[i] = (__bf16)a;
    r[4 + i] = (__bf16)b;
  }
  return r;
}

// 16-byte global loads of one 64 x D bf16 tile into registers (rows past `valid` read as zero),
// and the matching stores into a padded LDS tile.  NT threads cooperate.
template <int D, int NT>
struct TileRegs {
  static constexpr int kLoads = kTileTokens * TileGeom<D>::kChunksPerRow / NT;
  uint4 r[kLoads];
  __device__ __forceinline__ void load(const uint16_t* src /* first row of the tile */, int valid, int tid) {
#pragma unroll
    for (int i = 0; i < kLoads; i++) {
      int idx = tid + NT * i;
      int row = idx / TileGeom<D>::kChunksPerRow, ch = idx % TileGeom<D>::kChunksPerRow;
      r[i] = row < valid ? *reinterpret_cast<const uint4*>(src + (size_t)row * D + 8 * ch) : make_uint4(0, 0, 0, 0);
    }
  }
  __device__ __forceinline__ void store(uint16_t* tile, int tid) const {
#pragma unroll
    for (int i = 0; i < kLoads; i++) {
      int idx = tid + NT * i;
      int row = idx / TileGeom<D>::kChunksPerRow, ch = idx % TileGeom<D>::kChunksPerRow;
      *reinterpret_cast<uint4*>(tile + row * TileGeom<D>::kLd + 8 * ch) = r[i];
    }
  }
};

}  // namespace sla2
