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
#include <type_traits>

#include "common.h"

namespace sla2 {

constexpr int kTileTokens = 64;                    // b_kv
constexpr int kXcds = 8;                           // L2 domains; workgroups are dealt to them round-robin
constexpr int kVmcnt0 = 0x0F70;                    // s_waitcnt vmcnt(0), other counters untouched

// lanes l and l ^ 32 combine their values; both get the same bits
__device__ __forceinline__ float half_sum(float x) { return x + __shfl_xor(x, 32); }
__device__ __forceinline__ float half_max(float x) { return fmaxf(x, __shfl_xor(x, 32)); }

__device__ __forceinline__ f32x16 mfma_bf16(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// ---- LDS layouts of a 64-token tile of bf16 rows --------------------------------------------------
// Padded: rows of D + 8 elements (written with ordinary LDS stores).
// Swizzled: rows of exactly D elements whose 16-byte chunks are XOR-permuted by the row index.  This
// is the layout for tiles that the load unit writes straight into LDS (global_load_lds_dwordx4 puts
// lane l's 16 bytes at base + 16 l, so a tile has to be contiguous); the permutation is applied by
// choosing which global chunk a lane fetches, and keeps both the row-wise 16-byte operand reads and
// the transposing 8-byte reads spread over the banks.
template <int D> struct PaddedLayout {
  static constexpr int kRowElems = D + 8;
  static constexpr int kTileBytes = kTileTokens * kRowElems * 2;
  __device__ static __forceinline__ int offset(int row, int col) { return row * kRowElems + col; }   // elements
};
template <int D> struct SwizzledLayout {
  static constexpr int kChunks = D / 8;              // 16-byte chunks per row
  static constexpr int kRowElems = D;
  static constexpr int kTileBytes = kTileTokens * D * 2;
  __device__ static __forceinline__ int swz(int row) { return kChunks >= 16 ? 2 * (row & 7) : (row & 7); }
  __device__ static __forceinline__ int offset(int row, int col) {
    return row * D + (((col >> 3) ^ swz(row)) << 3) + (col & 7);
  }
};

// The same with a permutation that also serves the transposing 8-byte reads without bank conflicts (16 chunks
// per row only).  The row-wise 16-byte read of 16 consecutive rows needs 16 different chunk positions, so the
// permutation is a bijection of row % 16; the transposing read touches 4 consecutive rows x 4 consecutive
// chunks at a time and needs those 16 positions different as well, which the two low row bits provide by
// moving the chunk by multiples of 4:  position = chunk ^ (4 (row % 4) + (row / 4) % 4).
template <int D> struct SwizzledLayoutB {
  static_assert(D == 128, "16 chunks of 16 bytes per row");
  static constexpr int kChunks = 16;
  static constexpr int kRowElems = D;
  static constexpr int kTileBytes = kTileTokens * D * 2;
  __device__ static __forceinline__ int swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }
  __device__ static __forceinline__ int offset(int row, int col) {
    return row * D + (((col >> 3) ^ swz(row)) << 3) + (col & 7);
  }
};

template <int D> struct TileGeom {
  static constexpr int kLd = D + 8;                // bf16 elements per padded LDS row
  static constexpr int kChunksPerRow = D / 8;      // 16-byte chunks per row
};

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// 4 tokens x 16 channels per 16-lane group, transposed on the way out of LDS: on return lane l
// holds tile[row0 + 0..3][col0 + l % 32] (row0 may differ between the two lane halves).
template <class L>
__device__ __forceinline__ s16x4 read_tr4(const uint16_t* tile, int row0, int col0, int lane) {
  const int row = row0 + (lane % 16) / 4;
  const int col = col0 + 16 * ((lane / 16) % 2) + 4 * (lane % 4);
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(tile + L::offset(row, col)));
}

// V fragment in token order: lane l <- V[token(ks, l/32, 0..7)][col0 + l % 32]   (raw bf16 bits)
template <class L>
__device__ __forceinline__ bf16x8 v_fragment(const uint16_t* vtile, int ks, int col0, int lane) {
  const int g = lane / 32;
  s16x4 lo = read_tr4<L>(vtile, 16 * ks + 4 * g, col0, lane);
  s16x4 hi = read_tr4<L>(vtile, 16 * ks + 8 + 4 * g, col0, lane);
  typedef __attribute__((ext_vector_type(8))) short s16x8;
  s16x8 r = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, r);
}

// The same read with the contraction index in natural order: lane l <- tile[16 ks + 8 (l/32) + 0..7][col0 + l % 32]
template <class L>
__device__ __forceinline__ bf16x8 nat_fragment(const uint16_t* tile, int ks, int col0, int lane) {
  const int g = lane / 32;
  s16x4 lo = read_tr4<L>(tile, 16 * ks + 8 * g, col0, lane);
  s16x4 hi = read_tr4<L>(tile, 16 * ks + 8 * g + 4, col0, lane);
  typedef __attribute__((ext_vector_type(8))) short s16x8;
  s16x8 r = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, r);
}

// Row-wise operand fragment: lane l <- tile[row][col .. col + 7]  (one 16-byte read)
template <class L>
__device__ __forceinline__ bf16x8 row_fragment(const uint16_t* tile, int row, int col) {
  return *reinterpret_cast<const bf16x8*>(tile + L::offset(row, col));
}

// One 64 x D bf16 tile, global memory -> LDS without passing through registers.  NW waves cooperate;
// each global_load_lds_dwordx4 moves 1 KB (64 lanes x 16 bytes) into consecutive LDS bytes.
// Completion is counted by vmcnt.  Rows past `valid` (ragged last tile) repeat the last row.  One
// straight-line sequence for full and ragged tiles alike: the number of transfers in flight is then
// the same on every path, which lets later waits be counted instead of draining everything.
template <int D, int NW, class L = SwizzledLayout<D>>
__device__ __forceinline__ void dma_tile(const uint16_t* src /* first row */, int row_stride /* elements */, int valid,
                                         uint16_t* tile, int w, int lane) {
  constexpr int kRowsPerInstr = 1024 / (D * 2);
  constexpr int kInstrs = kTileTokens / kRowsPerInstr / NW;
  static_assert((kRowsPerInstr * NW) % 16 == 0 || (std::is_same<L, SwizzledLayout<D>>::value && (kRowsPerInstr * NW) % 8 == 0),
                "row swizzle must repeat between the instructions of a wave");
  const int row_w = w * kRowsPerInstr + lane / L::kChunks;           // row of instruction 0
  const unsigned col_bytes = 16u * (unsigned)((lane % L::kChunks) ^ L::swz(row_w));
  const char* base = reinterpret_cast<const char*>(src);
#pragma unroll
  for (int i = 0; i < kInstrs; i++) {
    const unsigned off = (unsigned)min(row_w + i * NW * kRowsPerInstr, valid - 1) * (unsigned)(row_stride * 2) + col_bytes;
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(base + off),
                                     (__attribute__((address_space(3))) void*)(tile + (i * NW + w) * 512), 16, 0, 0);
  }
}

// The same for a tile whose 64 rows all exist: no clamping, and every address is a per-lane constant
// plus a multiple of the instruction stride, which keeps the per-tile address arithmetic scalar.
template <int D, int NW>
__device__ __forceinline__ void dma_tile_full(const uint16_t* src, int row_stride /* elements */, uint16_t* tile, int w,
                                              int lane) {
  typedef SwizzledLayout<D> L;
  constexpr int kRowsPerInstr = 1024 / (D * 2);
  constexpr int kInstrs = kTileTokens / kRowsPerInstr / NW;
  const int row_w = w * kRowsPerInstr + lane / L::kChunks;
  const unsigned lane_off = (unsigned)row_w * (unsigned)(row_stride * 2) + 16u * (unsigned)((lane % L::kChunks) ^ L::swz(row_w));
  const char* base = reinterpret_cast<const char*>(src);
#pragma unroll
  for (int i = 0; i < kInstrs; i++)
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)(base + (size_t)i * (size_t)(NW * kRowsPerInstr * row_stride * 2) + lane_off),
        (__attribute__((address_space(3))) void*)(tile + (i * NW + w) * 512), 16, 0, 0);
}

// The same for a 64 x D tile of e4m3 codes.  Rows of D bytes; the operand of the 64-deep FP8
// product is 32 consecutive codes of a row, so the unit that is XOR-permuted is the aligned
// 32-byte pair of chunks (two 16-byte reads per operand, second at +16).
template <int D> struct SwizzledLayout8 {
  static constexpr int kChunks = D / 16;             // 16-byte chunks per row
  static constexpr int kPairs = D / 32;
  static constexpr int kTileBytes = kTileTokens * D;
  __device__ static __forceinline__ int swz(int row) { return (row >> 1) & (kPairs - 1); }
  __device__ static __forceinline__ int offset(int row, int col) {   // bytes
    return row * D + (((col >> 5) ^ swz(row)) << 5) + (col & 31);
  }
};
template <int D, int NW>
__device__ __forceinline__ void dma_tile8(const uint8_t* src, uint8_t* tile, int w, int lane) {
  typedef SwizzledLayout8<D> L;
  constexpr int kRowsPerInstr = 1024 / D;
  constexpr int kInstrs = kTileTokens / kRowsPerInstr / NW;
  static_assert(kInstrs >= 1 && (kRowsPerInstr * NW) % 8 == 0, "unsupported tile split");
  const int row_w = w * kRowsPerInstr + lane / L::kChunks;
  const int pc = lane % L::kChunks;                  // chunk slot this lane fills; it fetches the chunk that belongs there
  const int chunk = 2 * ((pc >> 1) ^ L::swz(row_w)) + (pc & 1);
  const uint8_t* g = src + row_w * D + 16 * chunk;
#pragma unroll
  for (int i = 0; i < kInstrs; i++)
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(g + i * NW * kRowsPerInstr * D),
                                     (__attribute__((address_space(3))) void*)(tile + (i * NW + w) * 1024), 16, 0, 0);
}

// A d x 64 tile of e4m3 codes of V, channel-major (rows of 64 bytes = the 64 tokens of a key block in
// the order the 64-deep product consumes them).  An operand is the 32 bytes of one half of a row,
// read as two 16-byte chunks; the chunk index is XOR-ed with (row / 4) % 4 so that the 16 rows one
// read instruction covers per lane group spread over all banks.
template <int D> struct SwizzledLayoutVq {
  static constexpr int kTileBytes = D * kTileTokens;
  __device__ static __forceinline__ int swz(int row) { return (row >> 2) & 3; }
  __device__ static __forceinline__ int offset(int row, int chunk) { return row * kTileTokens + ((chunk ^ swz(row)) << 4); }
};
template <int D, int NW>
__device__ __forceinline__ void dma_tile_vq(const uint8_t* src, uint8_t* tile, int w, int lane) {
  typedef SwizzledLayoutVq<D> L;
  constexpr int kRowsPerInstr = 1024 / kTileTokens;           // 16 rows of 64 bytes per instruction
  constexpr int kInstrs = D / kRowsPerInstr / NW;
  static_assert(kInstrs >= 1, "unsupported tile split");
#pragma unroll
  for (int i = 0; i < kInstrs; i++) {
    const int row = (i * NW + w) * kRowsPerInstr + lane / 4;  // the slot this lane fills holds chunk (lane % 4) ^ swz(row)
    const uint8_t* g = src + row * kTileTokens + 16 * ((lane % 4) ^ L::swz(row));
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                     (__attribute__((address_space(3))) void*)(tile + (i * NW + w) * 1024), 16, 0, 0);
  }
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// K^phi fragment in token order for channel col0 + l % 32:
//   K^phi[t][c] = exp(k[t][c] - mu[c] - lnZ[t]) = exp2(k log2e - (mu2 + lnz2[t]))
// lnz2: LDS array of 64 floats, lnZ[t] * log2e, +inf for tokens past the end (-> K^phi = 0).
// Adds the 8 fp32 values to zsum (column sums of K^phi, Alg. 2's z).
template <class L>
__device__ __forceinline__ bf16x8 kphi_fragment(const uint16_t* ktile, const float* lnz2, float mu2, int ks, int col0,
                                                int lane, float& zsum) {
  const int g = lane / 32;
  s16x4 lo = read_tr4<L>(ktile, 16 * ks + 4 * g, col0, lane);
  s16x4 hi = read_tr4<L>(ktile, 16 * ks + 8 + 4 * g, col0, lane);
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

// 16-byte global loads of one 64 x D bf16 tile into registers and the matching stores into a padded
// LDS tile.  NT threads cooperate.  Rows past `valid` repeat the last existing row: the loads stay
// unpredicated, so they can remain in flight across a whole compute phase.
template <int D, int NT> struct TileCopy {
  static constexpr int kLoads = kTileTokens * TileGeom<D>::kChunksPerRow / NT;
  __device__ static __forceinline__ void load(u32x4 (&r)[kLoads], const uint16_t* src /* first row */,
                                              int row_stride /* elements */, int valid, int tid) {
#pragma unroll
    for (int i = 0; i < kLoads; i++) {
      const int idx = tid + NT * i;
      const int row = min(idx / TileGeom<D>::kChunksPerRow, valid - 1), ch = idx % TileGeom<D>::kChunksPerRow;
      r[i] = *reinterpret_cast<const u32x4*>(src + (size_t)row * row_stride + 8 * ch);
    }
  }
  __device__ static __forceinline__ void store(const u32x4 (&r)[kLoads], uint16_t* tile, int tid) {
#pragma unroll
    for (int i = 0; i < kLoads; i++) {
      const int idx = tid + NT * i;
      const int row = idx / TileGeom<D>::kChunksPerRow, ch = idx % TileGeom<D>::kChunksPerRow;
      *reinterpret_cast<u32x4*>(tile + row * TileGeom<D>::kLd + 8 * ch) = r[i];
    }
  }
};

// A global load the compiler does not track: no wait is generated for it, the caller waits with
// wait_vmcnt<>() and then passes every loaded value through settle() before using it.  The load and the
// wait are compiler-level memory barriers ("memory" clobber): no other memory operation - in particular no
// global -> LDS transfer, which shares the vmcnt counter - can be moved across them, so the number of
// operations in flight between a load and its wait is the number written in the source.
template <class T>
__device__ __forceinline__ T load_untracked(const void* p) {
  T r;
  if constexpr (sizeof(T) == 16) asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(r) : "v"(p) : "memory");
  else asm volatile("global_load_dword %0, %1, off" : "=v"(r) : "v"(p) : "memory");
  return r;
}
template <class T, bool UNTRACKED>
__device__ __forceinline__ T load_maybe_tracked(const void* p) {
  if constexpr (UNTRACKED) return load_untracked<T>(p);
  else return *reinterpret_cast<const T*>(p);
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// Orders every later use of x after the preceding wait (volatile statements keep their order).
template <class T>
__device__ __forceinline__ void settle(T& x) { asm volatile("" : "+v"(x)); }

// LDS operand reads issued the same way.  The compiler's scheduler keeps a tracked read, its wait
// and the product that consumes it back to back, so the LDS latency is paid once per product; with
// the reads untracked the kernel keeps several in flight and waits with the count it knows.  The
// LDS counter retires in order, so "at most n outstanding" settles everything but the n youngest.
// Another benefit: a tracked transposing read is treated as a possible alias of the tile transfer
// in flight and is preceded by vmcnt(0).
__device__ __forceinline__ unsigned lds_address(const void* p) {
  return (unsigned)(size_t)(const __attribute__((address_space(3))) void*)p;
}
template <int OFF1>   // 8 bytes at addr and 8 bytes at addr + 512 OFF1
__device__ __forceinline__ u32x4 lds_read2_untracked(unsigned addr) {
  u32x4 r;
  asm volatile("ds_read2st64_b64 %0, %1 offset1:%2" : "=v"(r) : "v"(addr), "n"(OFF1));
  return r;
}
template <int OFF>    // 16 bytes at addr + OFF
__device__ __forceinline__ u32x4 lds_read16_untracked(unsigned addr) {
  u32x4 r;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
  return r;
}
template <int UNIT>   // 16 bytes at addr + n UNIT, the offset in the instruction (n constant after unrolling)
__device__ __forceinline__ u32x4 lds_read16_untracked_at(unsigned addr, int n) {
  switch (n) {
    case 0: return lds_read16_untracked<0>(addr);
    case 1: return lds_read16_untracked<UNIT>(addr);
    case 2: return lds_read16_untracked<2 * UNIT>(addr);
    default: return lds_read16_untracked<3 * UNIT>(addr);
  }
}
template <int OFF>    // transposing read, see read_tr4
__device__ __forceinline__ u32x2 lds_read_tr_untracked(unsigned addr) {
  u32x2 r;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
  return r;
}
// at addr + n UNIT with the offset in the instruction; n is a constant after unrolling
template <int UNIT>
__device__ __forceinline__ u32x2 lds_read_tr_untracked_at(unsigned addr, int n) {
  switch (n) {
    case 0: return lds_read_tr_untracked<0>(addr);
    case 1: return lds_read_tr_untracked<UNIT>(addr);
    case 2: return lds_read_tr_untracked<2 * UNIT>(addr);
    case 3: return lds_read_tr_untracked<3 * UNIT>(addr);
    case 4: return lds_read_tr_untracked<4 * UNIT>(addr);
    case 5: return lds_read_tr_untracked<5 * UNIT>(addr);
    case 6: return lds_read_tr_untracked<6 * UNIT>(addr);
    default: return lds_read_tr_untracked<7 * UNIT>(addr);
  }
}
// n is a constant once the calling loop is unrolled; only the matching statement survives
__device__ __forceinline__ void wait_lgkmcnt(int n) {
  switch (n) {
    case 0: asm volatile("s_waitcnt lgkmcnt(0)"); break;
    case 1: asm volatile("s_waitcnt lgkmcnt(1)"); break;
    case 2: asm volatile("s_waitcnt lgkmcnt(2)"); break;
    case 3: asm volatile("s_waitcnt lgkmcnt(3)"); break;
    case 4: asm volatile("s_waitcnt lgkmcnt(4)"); break;
    case 5: asm volatile("s_waitcnt lgkmcnt(5)"); break;
    case 6: asm volatile("s_waitcnt lgkmcnt(6)"); break;
    case 7: asm volatile("s_waitcnt lgkmcnt(7)"); break;
    case 8: asm volatile("s_waitcnt lgkmcnt(8)"); break;
    case 9: asm volatile("s_waitcnt lgkmcnt(9)"); break;
    case 10: asm volatile("s_waitcnt lgkmcnt(10)"); break;
    case 11: asm volatile("s_waitcnt lgkmcnt(11)"); break;
    case 12: asm volatile("s_waitcnt lgkmcnt(12)"); break;
    case 13: asm volatile("s_waitcnt lgkmcnt(13)"); break;
    case 14: asm volatile("s_waitcnt lgkmcnt(14)"); break;
    case 15: asm volatile("s_waitcnt lgkmcnt(15)"); break;
    default: asm volatile("s_waitcnt lgkmcnt(0)"); break;
  }
}

}  // namespace sla2
