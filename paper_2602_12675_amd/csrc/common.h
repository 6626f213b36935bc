// Shared declarations of the SLA2 HIP kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "../../include/sla2.h"

namespace sla2 {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) double f64x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;   // 16 bytes in flight (a native vector: stays in registers)
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
typedef __attribute__((ext_vector_type(8))) int i32x8;            // operand of the 64-deep FP8 product
typedef __attribute__((ext_vector_type(4))) int i32x4;            // operand of the 32-deep INT8 product
typedef __attribute__((ext_vector_type(16))) int i32x16;          // its 32 x 32 accumulator

constexpr int kWave = 64;
constexpr int kMaxKeyBlocks = 2048;   // router keeps a whole score row in registers
constexpr float kE4M3Max = 448.0f;
constexpr float kInt8Max = 127.0f;   // symmetric INT8 code range of Q and K
constexpr float kLog2e = 1.4426950408889634f;

// Where (batch b, head h, token t) of a [.., d] tensor starts, in elements: b * b_ + h * h_ + t * n.
struct Strides {
  long long b, h;
  int n;
};
__host__ __device__ __forceinline__ size_t head_offset(const Strides& st, int bh, int H) {
  return (size_t)(bh / H) * (size_t)st.b + (size_t)(bh % H) * (size_t)st.h;
}

// hipFuncSetAttribute(MaxDynamicSharedMemorySize) once per kernel and device.  Safe to call from several
// threads: the flag is atomic and setting the attribute twice is harmless.
struct OncePerDevice { std::atomic<unsigned long long> done{0}; };
inline hipError_t allow_dynamic_lds(OncePerDevice& once, const void* kernel, int bytes) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const unsigned long long bit = 1ull << (dev & 63);
  if (once.done.load(std::memory_order_acquire) & bit) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) once.done.fetch_or(bit, std::memory_order_release);
  return e;
}

// Host-side description of one call, derived from sla2_params.
struct Shape {
  Strides sin, sout;                         // q, k, v share `sin`; out has `sout`
  int B, H, N, d, bq, bk;
  int BH, Tm, Tn, k;
  bool bf16, smooth, w_per_head, alpha_per_block;
  bool save;                                 // keep O^s, O^l, L for the backward pass
  int quant;                                 // sla2_quant: 0 none, 1 FP8 e4m3, 2 INT8 codes of Q and K, 3 FP8 with V in e4m3 too
  // kv precompute: each workgroup reduces `blocks_per_chunk` key blocks; `chunks` per head
  int blocks_per_chunk, chunks;
};

// sla2_api.cpp: parameter validation (SLA2_OK or a negative sla2_status) and the workspace carve-up
int make_shape(const sla2_params* p, Shape* s);
void make_layout(const Shape& s, sla2_ws_layout* L);

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) {
  return __builtin_bit_cast(float, (uint32_t)b << 16);
}
// round to nearest even; inputs are finite
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float load_elem(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_elem(const uint16_t* p, size_t i) { return bf16_bits_to_f32(p[i]); }
__device__ __forceinline__ void store_elem(float* p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void store_elem(uint16_t* p, size_t i, float v) { p[i] = f32_to_bf16_bits(v); }

// Where sla2_forward keeps O^s, O^l ([BH, N, d], element type of out; o_l may be null on its own) and
// L ([BH, N]) for the backward pass; all null when nothing is to be kept.  The bf16 kernels also keep the state of the linear branch
// per query block: H_i^T as bf16 [BH, T_m, d(e), d(c)] and Z_i [BH, T_m, d] (null for fp32 tensors, whose
// backward pass rebuilds them).
struct SavedForBackward {
  void *o_s, *o_l;
  float* lse;
  uint16_t* h_i;
  float* z_i;
};

// Everything the backward kernels touch (device pointers).
struct BwdArgs {
  const void *q, *k, *v, *dout, *o_s, *o_l;
  const float* lse;
  const double* k_mean;
  const float *k_stats, *h_total, *z_total;
  const int32_t* block_idx;
  const float* alpha;
  void *dq, *dk, *dv;
  float* dalpha;
  // kept by the bf16 forward kernel: H_i^T as bf16 [BH, T_m, d, d], Z_i [BH, T_m, d]
  const uint16_t* h_i;
  const float* z_i;
  // scratch.  dh: one d x d slot per query block as bf16 (bf16 tensors) or per 64 query rows as fp32
  float *ds, *lraw, *dz, *dh_total, *dz_total, *colsum, *dk_mean, *dalpha_part;
  void* dh;
  int32_t *col_ptr, *col_idx, *col_cnt;
  uint32_t* mask_bits;                       // M_c as bits, [BH, T_m, ceil(T_n / 32)]
};
// the backward pass in the order it runs: lists, query side, totals, key side, finish
hipError_t launch_bwd_lists(const Shape& s, const BwdArgs& a, hipStream_t stream);
hipError_t launch_bwd_q(const Shape& s, const BwdArgs& a, hipStream_t stream);
hipError_t launch_bwd_totals(const Shape& s, const BwdArgs& a, hipStream_t stream);
hipError_t launch_bwd_kv(const Shape& s, const BwdArgs& a, hipStream_t stream);
hipError_t launch_bwd_finish(const Shape& s, const BwdArgs& a, hipStream_t stream);
hipError_t launch_bwd_q_bf16(const Shape& s, const BwdArgs& a, hipStream_t stream);   // matrix-core kernels, bf16 tensors
hipError_t launch_bwd_kv_bf16(const Shape& s, const BwdArgs& a, hipStream_t stream);

// ---- launchers (one per kernel file); all enqueue on `stream` and return hipGetLastError() ----
hipError_t launch_block_sums(const Shape& s, const void* q, const void* k, const float* router_w, double* q_sum,
                             double* k_sum, double* router_m, hipStream_t stream);
hipError_t launch_router_topk(const Shape& s, const double* q_sum, const double* k_sum, const double* router_m,
                              int32_t* block_idx, double* k_mean, hipStream_t stream);
hipError_t launch_router_soft(const Shape& s, const double* q_sum, const double* k_sum, const double* router_m,
                              float* mask, double tau, hipStream_t stream);
hipError_t launch_kv_state_f32(const Shape& s, const float* k, const float* v, const double* k_mean, float* k_stats,
                               float* partial, hipStream_t stream);
hipError_t launch_attn_f32(const Shape& s, const float* q, const float* k, const float* v, const double* k_mean,
                           const float* k_stats, const float* h_total, const float* z_total, const int32_t* block_idx,
                           const float* alpha, float* out, float* lse, const SavedForBackward& sv, hipStream_t stream);

hipError_t launch_kv_total(const Shape& s, const float* partial, float* h_total, float* z_total, hipStream_t stream);
hipError_t launch_kv_state_bf16(const Shape& s, const uint16_t* k, const uint16_t* v, const double* k_mean,
                                float* k_stats, float* partial, uint16_t* k_phi, float* z_blocks, uint8_t* k_codes,
                                float* k_scale, uint8_t* v_codes, float* v_scale, hipStream_t stream);
hipError_t launch_attn_bf16(const Shape& s, const uint16_t* q, const uint16_t* k, const uint16_t* v,
                            const double* k_mean, const uint16_t* k_phi, const float* z_blocks, const uint8_t* k_codes,
                            const float* k_scale, const uint8_t* v_codes, const float* v_scale,
                            const float* h_total, const float* z_total,
                            const int32_t* block_idx, const float* alpha, uint16_t* out, float* lse,
                            const SavedForBackward& sv, hipStream_t stream);
hipError_t launch_dense_pp(const Shape& s, const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* out,
                           hipStream_t stream);
hipError_t launch_dense_bf16(const Shape& s, const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* out,
                             hipStream_t stream);

}  // namespace sla2
