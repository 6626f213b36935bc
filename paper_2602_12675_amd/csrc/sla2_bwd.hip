// Backward pass of SLA2 (Alg. 3 of the paper's appendix, with the steps it leaves to automatic
// differentiation written out: phi = softmax over d, the smoothing of K, the mix of Eq. 13).
// High precision throughout, from the original Q, K, V (Sec. 5: the backward pass is never quantised).
//
// This file holds the launch sequence, the small kernels every tensor type shares, and the two heavy
// kernels for fp32 tensors: plain LDS-tiled FMA kernels in fp32 - the readable, deterministic
// statement of the data flow (no atomics, fixed summation orders); they are not tuned.  bf16 tensors
// run the two heavy steps on the matrix cores instead (sla2_bwd_mfma.hip).
//
//   bwd_mask_bits, bwd_col_count / _scan / _fill
//                  M_c as bits, then for every key block j the ascending list of query blocks i with
//                  M_c[i, j] = 1
//   bwd_q          per 64 query rows of block i:  D^s, D^l, d alpha;  over the selected blocks:
//                  P = exp(S - L), dP = dO^s V^T, dS = P (.) (dP - D^s), dQ += dS K' / sqrt d, and the
//                  state of the selected blocks (as in the forward pass) -> H_i, Z_i;  then
//                  dH_i = (Q^phi / (Q^phi Z_i))^T dO^l, dZ_i, dQ^phi, dQ += softmax-backward(dQ^phi)
//   bwd_sum        dH_total = sum_i dH_i, dZ_total = sum_i dZ_i
//   bwd_kv         per key block j:  over the query blocks that selected it: dV += P^T dO^s,
//                  dK' += dS^T Q / sqrt d;  dH = dH_total - sum over those same query blocks of dH_i
//                  (the M_c[i, j] = 0 sum of Alg. 3, by complement), dZ likewise;
//                  dK^phi = V dH^T + 1 dZ^T, dV += K^phi dH, dK' += softmax-backward(dK^phi)
//   bwd_colmean, bwd_unsmooth, bwd_dalpha
//                  dK = dK' - colmean(dK') (gradient of the smoothing), d alpha summed over its parts
#include "common.h"

namespace sla2 {

constexpr int kBwdRows = 64;      // query rows per workgroup / per step
constexpr int kBwdBK = 64;        // key/value block (b_kv)

// ---------------------------------------------------------------------------------------------
// M_c as bits: row (bh, i) -> ceil(T_n / 32) words, bit j % 32 of word j / 32 set iff block j is selected
__global__ __launch_bounds__(64) void bwd_mask_bits_kernel(const int32_t* __restrict__ block_idx,
                                                           uint32_t* __restrict__ bits, int Tn, int ksel) {
  __shared__ uint32_t words[kMaxKeyBlocks / 32];
  const int W = (Tn + 31) / 32, tid = threadIdx.x;
  for (int x = tid; x < W; x += 64) words[x] = 0u;
  __syncthreads();
  const int32_t* row = block_idx + (size_t)blockIdx.x * ksel;
  for (int s = tid; s < ksel; s += 64) {
    const int j = row[s];
    atomicOr(&words[j >> 5], 1u << (j & 31));         // OR: the result does not depend on the order
  }
  __syncthreads();
  for (int x = tid; x < W; x += 64) bits[(size_t)blockIdx.x * W + x] = words[x];
}

// For every key block j of head bh: the ascending list of query blocks i with M_c[i, j] = 1, as
// offsets col_ptr[bh][0..T_n] into col_idx[bh][.].  Three small kernels: column counts, their
// exclusive scan, and the fill.  Counts and fill run one wave per (head, 32-column word): the wave
// walks the bit rows 64 at a time, one ballot per column; the rank of a set bit inside the ballot
// plus the running count of the column is its place in the (ascending) list.
__global__ __launch_bounds__(64) void bwd_col_count_kernel(const uint32_t* __restrict__ bits, int32_t* __restrict__ counts,
                                                           int Tm, int Tn) {
  const int W = (Tn + 31) / 32, x = blockIdx.x, bh = blockIdx.y, lane = threadIdx.x;
  const uint32_t* rows = bits + (size_t)bh * Tm * W + x;
  int run[32];
#pragma unroll
  for (int b = 0; b < 32; b++) run[b] = 0;
  for (int i0 = 0; i0 < Tm; i0 += 64) {
    const int i = i0 + lane;
    const uint32_t word = i < Tm ? rows[(size_t)i * W] : 0u;
#pragma unroll
    for (int b = 0; b < 32; b++) run[b] += __popcll(__ballot((word >> b) & 1u));
  }
  int mine = 0;
#pragma unroll
  for (int b = 0; b < 32; b++) mine = lane == b ? run[b] : mine;
  const int j = 32 * x + lane;
  if (lane < 32 && j < Tn) counts[(size_t)bh * Tn + j] = mine;
}

__global__ __launch_bounds__(256) void bwd_col_scan_kernel(const int32_t* __restrict__ counts, int32_t* __restrict__ col_ptr,
                                                           int Tn) {
  constexpr int PER = kMaxKeyBlocks / 256;
  __shared__ int part[256];
  const int bh = blockIdx.x, tid = threadIdx.x;
  int v[PER], sum = 0;
#pragma unroll
  for (int y = 0; y < PER; y++) {
    const int j = tid * PER + y;
    v[y] = j < Tn ? counts[(size_t)bh * Tn + j] : 0;
    sum += v[y];
  }
  part[tid] = sum;
  __syncthreads();
  if (tid == 0) {                                     // exclusive scan of the 256 partial sums, in place
    int run = 0;
    for (int t = 0; t < 256; t++) {
      const int c = part[t];
      part[t] = run;
      run += c;
    }
  }
  __syncthreads();
  int run = part[tid];
#pragma unroll
  for (int y = 0; y < PER; y++) {
    const int j = tid * PER + y;
    if (j < Tn) col_ptr[(size_t)bh * (Tn + 1) + j] = run;
    run += v[y];
    if (j == Tn - 1) col_ptr[(size_t)bh * (Tn + 1) + Tn] = run;
  }
}

__global__ __launch_bounds__(64) void bwd_col_fill_kernel(const uint32_t* __restrict__ bits, const int32_t* __restrict__ col_ptr,
                                                          int32_t* __restrict__ col_idx, int Tm, int Tn, int ksel) {
  const int W = (Tn + 31) / 32, x = blockIdx.x, bh = blockIdx.y, lane = threadIdx.x;
  const uint32_t* rows = bits + (size_t)bh * Tm * W + x;
  int32_t* out = col_idx + (size_t)bh * Tm * ksel;
  int run[32];
#pragma unroll
  for (int b = 0; b < 32; b++) run[b] = 32 * x + b < Tn ? col_ptr[(size_t)bh * (Tn + 1) + 32 * x + b] : 0;
  const unsigned long long below = (1ull << lane) - 1ull;
  for (int i0 = 0; i0 < Tm; i0 += 64) {
    const int i = i0 + lane;
    const uint32_t word = i < Tm ? rows[(size_t)i * W] : 0u;
#pragma unroll
    for (int b = 0; b < 32; b++) {
      const unsigned long long m = __ballot((word >> b) & 1u);
      if ((word >> b) & 1u) out[run[b] + __popcll(m & below)] = i;
      run[b] += __popcll(m);
    }
  }
}

// sum over the 16 lanes that share a row (threads tx = 0..15 of one ty)
__device__ __forceinline__ float row_sum16(float v) {
#pragma unroll
  for (int o = 1; o < 16; o <<= 1) v += __shfl_xor(v, o);
  return v;
}

// ---------------------------------------------------------------------------------------------
// bwd_q: one workgroup per 64 query rows.  Thread (tx, ty): rows 4 ty + a, key tokens / channels
// tx + 16 b; for d x d quantities, entries (MT ty + a, tx + 16 b).
// ---------------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(256) void bwd_q_kernel(
    const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v, const T* __restrict__ dout,
    const T* __restrict__ o_s, const T* __restrict__ o_l, const float* __restrict__ lse,
    const double* __restrict__ k_mean, const float* __restrict__ k_stats, const float* __restrict__ h_total,
    const float* __restrict__ z_total, const int32_t* __restrict__ block_idx, const float* __restrict__ alpha,
    T* __restrict__ dq, float* __restrict__ ds_out, float* __restrict__ dh_out, float* __restrict__ dz_out,
    float* __restrict__ dalpha_part, Strides sin, Strides sout, int H, int N, int bq, int Tm, int Tn, int ksel,
    int alpha_per_block) {
  constexpr int LD = D + 1;
  constexpr int LP = kBwdBK + 1;
  constexpr int MT = D / 16;
  constexpr int OC = D / 16;
  extern __shared__ float smem[];
  float* qs = smem;                         // [64][LD]  Q rows, later Q^phi
  float* dos = qs + kBwdRows * LD;          // [64][LD]  dO^s rows, later dO^l rows
  float* ks = dos + kBwdRows * LD;          // [64][LD]  K' tile, then K^phi tile
  float* vs = ks + kBwdBK * LD;             // [64][LD]  V tile
  float* ps = vs + kBwdBK * LD;             // [64][LP]  dS tile
  float* zs = ps + kBwdRows * LP;           // [D]       Z_i
  float* rowv = zs + D;                     // [64]      1 / (Q^phi Z_i) per row
  float* rowd = rowv + kBwdRows;            // [64]      D^l per row
  float* red = rowd + kBwdRows;             // [256]
  float* hst = ks;                          // [D][D]    H_i^T in the epilogue (covers ks and vs)

  const int parts = bq / kBwdRows;
  int bid = blockIdx.x;
  const int part = bid % parts; bid /= parts;
  const int i = bid % Tm;
  const int bh = bid / Tm;
  const int h = bh % H;
  const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
  const int row0 = i * bq + part * kBwdRows;
  const int rows_valid = max(0, min(kBwdRows, min(N, (i + 1) * bq) - row0));
  const size_t slot = ((size_t)bh * Tm + i) * parts + part;          // where this workgroup's dH_i, dZ_i, d alpha go
  float* dh_slot = dh_out + slot * D * D;
  float* dz_slot = dz_out + slot * D;
  if (rows_valid == 0) {                                              // second half of a short last query block
    for (int e = tid; e < D * D; e += 256) dh_slot[e] = 0.f;
    if (tid < D) dz_slot[tid] = 0.f;
    if (tid == 0) dalpha_part[slot] = 0.f;
    return;
  }
  const T* qh = q + head_offset(sin, bh, H);
  const T* kh = k + head_offset(sin, bh, H);
  const T* vh = v + head_offset(sin, bh, H);
  const T* doh = dout + head_offset(sout, bh, H);
  T* dqh = dq + head_offset(sin, bh, H);
  const int32_t* sel = block_idx + ((size_t)bh * Tm + i) * ksel;
  const float rscale = rsqrtf((float)D);
  const float al = alpha[alpha_per_block ? (size_t)h * Tm + i : (size_t)h];

  // ---- prologue: Q, dO^s = alpha dO; D^s, D^l, d alpha ----
  float Ds[4], Dl[4], Lr[4];
  float mix_part = 0.f;
#pragma unroll
  for (int a = 0; a < 4; a++) {
    const int r = 4 * ty + a;
    const bool ok = r < rows_valid;
    float sds = 0.f, sdl = 0.f;
#pragma unroll
    for (int b = 0; b < OC; b++) {
      const int c = tx + 16 * b;
      float qv = 0.f, go = 0.f, osv = 0.f, olv = 0.f;
      if (ok) {
        qv = load_elem(qh, (size_t)(row0 + r) * sin.n + c);
        go = load_elem(doh, (size_t)(row0 + r) * sout.n + c);
        osv = load_elem(o_s, ((size_t)bh * N + row0 + r) * D + c);
        olv = load_elem(o_l, ((size_t)bh * N + row0 + r) * D + c);
      }
      qs[r * LD + c] = qv;
      dos[r * LD + c] = al * go;
      sds += al * go * osv;
      sdl += (1.f - al) * go * olv;
      mix_part += go * (osv - olv);
    }
    Ds[a] = row_sum16(sds);
    Dl[a] = row_sum16(sdl);
    Lr[a] = ok ? lse[(size_t)bh * N + row0 + r] : 0.f;
    if (ok && tx == 0) ds_out[(size_t)bh * N + row0 + r] = Ds[a];
    if (tx == 0) rowd[r] = Dl[a];
  }
  red[tid] = mix_part;
  __syncthreads();
  if (tid == 0) {
    float t = 0.f;
    for (int x = 0; x < 256; x++) t += red[x];
    dalpha_part[slot] = t;
  }

  float dqacc[4][OC], hacc[MT][MT];
#pragma unroll
  for (int a = 0; a < 4; a++)
#pragma unroll
    for (int b = 0; b < OC; b++) dqacc[a][b] = 0.f;
#pragma unroll
  for (int a = 0; a < MT; a++)
#pragma unroll
    for (int b = 0; b < MT; b++) hacc[a][b] = 0.f;
  float zacc = 0.f;

  for (int s = 0; s < ksel; s++) {
    const int j = sel[s];
    const int t0 = j * kBwdBK, valid = min(kBwdBK, N - t0);
    __syncthreads();                                  // previous tile fully consumed
    for (int idx = tid; idx < kBwdBK * D; idx += 256) {
      const int t = idx / D, c = idx % D;
      const bool ok = t < valid;
      ks[t * LD + c] = ok ? load_elem(kh, (size_t)(t0 + t) * sin.n + c) - (float)k_mean[(size_t)bh * D + c] : 0.f;
      vs[t * LD + c] = ok ? load_elem(vh, (size_t)(t0 + t) * sin.n + c) : 0.f;
    }
    __syncthreads();
    // S = Q K'^T / sqrt d and dP = dO^s V^T on rows 4 ty + a, key tokens tx + 16 b
    float sacc[4][4], pacc[4][4];
#pragma unroll
    for (int a = 0; a < 4; a++)
#pragma unroll
      for (int b = 0; b < 4; b++) { sacc[a][b] = 0.f; pacc[a][b] = 0.f; }
    for (int c = 0; c < D; c++) {
      float qv[4], gv[4], kv[4], vv[4];
#pragma unroll
      for (int a = 0; a < 4; a++) { qv[a] = qs[(4 * ty + a) * LD + c]; gv[a] = dos[(4 * ty + a) * LD + c]; }
#pragma unroll
      for (int b = 0; b < 4; b++) { kv[b] = ks[(tx + 16 * b) * LD + c]; vv[b] = vs[(tx + 16 * b) * LD + c]; }
#pragma unroll
      for (int a = 0; a < 4; a++)
#pragma unroll
        for (int b = 0; b < 4; b++) { sacc[a][b] += qv[a] * kv[b]; pacc[a][b] += gv[a] * vv[b]; }
    }
#pragma unroll
    for (int a = 0; a < 4; a++)
#pragma unroll
      for (int b = 0; b < 4; b++) {
        const bool ok = (tx + 16 * b) < valid && (4 * ty + a) < rows_valid;
        const float p = ok ? __expf(sacc[a][b] * rscale - Lr[a]) : 0.f;
        ps[(4 * ty + a) * LP + tx + 16 * b] = p * (pacc[a][b] - Ds[a]);     // dS
      }
    __syncthreads();
    // dQ += dS K' / sqrt d
    for (int t = 0; t < kBwdBK; t++) {
      float sv[4], kv[OC];
#pragma unroll
      for (int a = 0; a < 4; a++) sv[a] = ps[(4 * ty + a) * LP + t];
#pragma unroll
      for (int b = 0; b < OC; b++) kv[b] = ks[t * LD + tx + 16 * b];
#pragma unroll
      for (int a = 0; a < 4; a++)
#pragma unroll
        for (int b = 0; b < OC; b++) dqacc[a][b] += sv[a] * kv[b];
    }
    __syncthreads();                                  // ks no longer read as K'
    for (int idx = tid; idx < kBwdBK * D; idx += 256) {
      const int t = idx / D, c = idx % D;
      float kp = 0.f;
      if (t < valid) kp = __expf(ks[t * LD + c] - k_stats[(size_t)bh * N + t0 + t]);
      ks[t * LD + c] = kp;
    }
    __syncthreads();
    for (int t = 0; t < kBwdBK; t++) {                // state of this selected block, as in the forward pass
      float kv[MT], vv[MT];
#pragma unroll
      for (int a = 0; a < MT; a++) kv[a] = ks[t * LD + MT * ty + a];
#pragma unroll
      for (int b = 0; b < MT; b++) vv[b] = vs[t * LD + tx + 16 * b];
#pragma unroll
      for (int a = 0; a < MT; a++)
#pragma unroll
        for (int b = 0; b < MT; b++) hacc[a][b] += kv[a] * vv[b];
    }
    if (tid < D)
      for (int t = 0; t < kBwdBK; t++) zacc += ks[t * LD + tid];
  }
  __syncthreads();

  // ---- linear branch ----
  const bool all_selected = ksel >= Tn;               // no linear branch: it receives and passes no gradient
  const float* ht = h_total + (size_t)bh * D * D;
#pragma unroll
  for (int a = 0; a < MT; a++)
#pragma unroll
    for (int b = 0; b < MT; b++) {
      const int c = MT * ty + a, e = tx + 16 * b;
      hst[e * D + c] = ht[c * D + e] - hacc[a][b];    // H_i^T: the product below runs over e
    }
  if (tid < D) zs[tid] = z_total[(size_t)bh * D + tid] - zacc;
  {  // Q^phi = softmax_d(Q) in place, 4 threads per row
    const int r = tid / 4, sub = tid % 4;
    float m = -INFINITY;
    for (int c = sub; c < D; c += 4) m = fmaxf(m, qs[r * LD + c]);
    m = fmaxf(m, __shfl_xor(m, 1));
    m = fmaxf(m, __shfl_xor(m, 2));
    float sum = 0.f;
    for (int c = sub; c < D; c += 4) {
      const float e = __expf(qs[r * LD + c] - m);
      qs[r * LD + c] = e;
      sum += e;
    }
    sum += __shfl_xor(sum, 1);
    sum += __shfl_xor(sum, 2);
    const float inv = 1.f / sum;
    for (int c = sub; c < D; c += 4) qs[r * LD + c] *= inv;
  }
  // dO^l = (1 - alpha) dO into the rows that held dO^s
  for (int idx = tid; idx < kBwdRows * D; idx += 256) {
    const int r = idx / D, c = idx % D;
    dos[r * LD + c] = r < rows_valid ? (1.f - al) * load_elem(doh, (size_t)(row0 + r) * sout.n + c) : 0.f;
  }
  __syncthreads();
  if (tid < kBwdRows) {                               // 1 / (Q^phi_r . Z_i)
    float den = 0.f;
    for (int c = 0; c < D; c++) den += qs[tid * LD + c] * zs[c];
    rowv[tid] = (all_selected || tid >= rows_valid) ? 0.f : 1.f / den;
  }
  __syncthreads();
  // dH_i[c][e] = sum_r (Q^phi[r][c] / den_r) dO^l[r][e];  dZ_i[c] = -sum_r (Q^phi[r][c] / den_r) D^l_r
  {
    float dh[MT][MT];
#pragma unroll
    for (int a = 0; a < MT; a++)
#pragma unroll
      for (int b = 0; b < MT; b++) dh[a][b] = 0.f;
    for (int r = 0; r < kBwdRows; r++) {
      const float w = rowv[r];
      float qv[MT], gv[MT];
#pragma unroll
      for (int a = 0; a < MT; a++) qv[a] = qs[r * LD + MT * ty + a] * w;
#pragma unroll
      for (int b = 0; b < MT; b++) gv[b] = dos[r * LD + tx + 16 * b];
#pragma unroll
      for (int a = 0; a < MT; a++)
#pragma unroll
        for (int b = 0; b < MT; b++) dh[a][b] += qv[a] * gv[b];
    }
#pragma unroll
    for (int a = 0; a < MT; a++)
#pragma unroll
      for (int b = 0; b < MT; b++) dh_slot[(MT * ty + a) * D + tx + 16 * b] = dh[a][b];
    if (tid < D) {
      float dzv = 0.f;
      for (int r = 0; r < kBwdRows; r++) dzv -= qs[r * LD + tid] * rowv[r] * rowd[r];
      dz_slot[tid] = dzv;
    }
  }
  // dQ^phi[r][c] = (sum_e dO^l[r][e] H_i[c][e] - D^l_r Z_i[c]) / den_r, then back through the softmax
  float dqp[4][OC];
#pragma unroll
  for (int a = 0; a < 4; a++)
#pragma unroll
    for (int b = 0; b < OC; b++) dqp[a][b] = 0.f;
  for (int e = 0; e < D; e++) {
    float gv[4], hv[OC];
#pragma unroll
    for (int a = 0; a < 4; a++) gv[a] = dos[(4 * ty + a) * LD + e];
#pragma unroll
    for (int b = 0; b < OC; b++) hv[b] = hst[e * D + tx + 16 * b];
#pragma unroll
    for (int a = 0; a < 4; a++)
#pragma unroll
      for (int b = 0; b < OC; b++) dqp[a][b] += gv[a] * hv[b];
  }
#pragma unroll
  for (int a = 0; a < 4; a++) {
    const int r = 4 * ty + a;
    const float w = rowv[r];
    float dot = 0.f;
#pragma unroll
    for (int b = 0; b < OC; b++) {
      const int c = tx + 16 * b;
      dqp[a][b] = (dqp[a][b] - Dl[a] * zs[c]) * w;
      dot += dqp[a][b] * qs[r * LD + c];
    }
    dot = row_sum16(dot);
    if (r < rows_valid) {
#pragma unroll
      for (int b = 0; b < OC; b++) {
        const int c = tx + 16 * b;
        const float g = dqacc[a][b] * rscale + qs[r * LD + c] * (dqp[a][b] - dot);
        store_elem(dqh, (size_t)(row0 + r) * sin.n + c, g);
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// dst[bh][e] = sum over b < count of src[bh][b][e].  A workgroup covers 256 consecutive e: 32 threads
// of 8 elements each, times 8 interleaved subsets of b that are combined in a fixed order.
template <typename S>
__global__ __launch_bounds__(256) void bwd_sum_kernel(const S* __restrict__ src, float* __restrict__ dst, int count,
                                                      int len) {
  __shared__ float part[8][256];
  const int bh = blockIdx.y, tid = threadIdx.x, col = tid % 32, sub = tid / 32;
  const int e0 = blockIdx.x * 256 + 8 * col;
  float acc[8];
#pragma unroll
  for (int x = 0; x < 8; x++) acc[x] = 0.f;
  if (e0 < len) {
    const S* p = src + (size_t)bh * count * len + e0;
#pragma unroll 4
    for (int b = sub; b < count; b += 8) {
      float v[8];
      if constexpr (sizeof(S) == 2) {
        const bf16x8 x = *reinterpret_cast<const bf16x8*>(p + (size_t)b * len);
#pragma unroll
        for (int y = 0; y < 8; y++) v[y] = (float)x[y];
      } else {
        const f32x4 x0 = *reinterpret_cast<const f32x4*>(p + (size_t)b * len), x1 = *reinterpret_cast<const f32x4*>(p + (size_t)b * len + 4);
#pragma unroll
        for (int y = 0; y < 4; y++) { v[y] = x0[y]; v[4 + y] = x1[y]; }
      }
#pragma unroll
      for (int y = 0; y < 8; y++) acc[y] += v[y];
    }
  }
#pragma unroll
  for (int x = 0; x < 8; x++) part[sub][8 * col + x] = acc[x];
  __syncthreads();
  const int e = blockIdx.x * 256 + tid;
  if (e < len) {
    float t = 0.f;
#pragma unroll
    for (int g = 0; g < 8; g++) t += part[g][tid];
    dst[(size_t)bh * len + e] = t;
  }
}

// ---------------------------------------------------------------------------------------------
// bwd_kv: one workgroup per key block j.  Thread (tx, ty): key tokens 4 ty + a, channels tx + 16 b;
// for the products over the 64 query rows of a step, rows tx + 16 b.
// ---------------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(256) void bwd_kv_kernel(
    const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v, const T* __restrict__ dout,
    const float* __restrict__ lse, const float* __restrict__ ds_in, const double* __restrict__ k_mean,
    const float* __restrict__ k_stats, const int32_t* __restrict__ col_ptr, const int32_t* __restrict__ col_idx,
    const float* __restrict__ dh_in, const float* __restrict__ dz_in, const float* __restrict__ dh_total,
    const float* __restrict__ dz_total, const float* __restrict__ alpha, T* __restrict__ dk, T* __restrict__ dv,
    float* __restrict__ colsum, Strides sin, Strides sout, int H, int N, int bq, int Tm, int Tn, int ksel,
    int alpha_per_block) {
  constexpr int LD = D + 1;
  constexpr int LP = kBwdBK + 1;
  constexpr int MT = D / 16;
  constexpr int OC = D / 16;
  extern __shared__ float smem[];
  float* ks = smem;                         // [64][LD]  K' tile, then K^phi tile
  float* vs = ks + kBwdBK * LD;             // [64][LD]  V tile
  float* qs = vs + kBwdBK * LD;             // [64][LD]  Q rows of the step
  float* dos = qs + kBwdRows * LD;          // [64][LD]  dO^s rows of the step
  float* ps = dos + kBwdRows * LD;          // [64 rows][LP]  P, then dS
  float* rowl = ps + kBwdRows * LP;         // [64]  L per row
  float* rowd = rowl + kBwdRows;            // [64]  D^s per row
  float* dzs = rowd + kBwdRows;             // [D]   dZ of this key block
  float* red = dzs + D;                     // [16][D] column sums
  float* dhs = qs;                          // [D][D]  dH, then dH^T, after the loop (covers qs and dos)

  const int j = blockIdx.x % Tn, bh = blockIdx.x / Tn, h = bh % H;
  const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
  const int t0 = j * kBwdBK, valid = min(kBwdBK, N - t0);
  const int parts = bq / kBwdRows;
  const T* qh = q + head_offset(sin, bh, H);
  const T* kh = k + head_offset(sin, bh, H);
  const T* vh = v + head_offset(sin, bh, H);
  const T* doh = dout + head_offset(sout, bh, H);
  const float rscale = rsqrtf((float)D);

  for (int idx = tid; idx < kBwdBK * D; idx += 256) {
    const int t = idx / D, c = idx % D;
    const bool ok = t < valid;
    ks[t * LD + c] = ok ? load_elem(kh, (size_t)(t0 + t) * sin.n + c) - (float)k_mean[(size_t)bh * D + c] : 0.f;
    vs[t * LD + c] = ok ? load_elem(vh, (size_t)(t0 + t) * sin.n + c) : 0.f;
  }
  float dvacc[4][OC], dkacc[4][OC];
#pragma unroll
  for (int a = 0; a < 4; a++)
#pragma unroll
    for (int b = 0; b < OC; b++) { dvacc[a][b] = 0.f; dkacc[a][b] = 0.f; }

  const int32_t* cp = col_ptr + (size_t)bh * (Tn + 1);
  const int32_t* ci = col_idx + (size_t)bh * Tm * ksel;
  const int l0 = cp[j], l1 = cp[j + 1];
  for (int l = l0; l < l1; l++) {
    const int i = ci[l];
    const float al = alpha[alpha_per_block ? (size_t)h * Tm + i : (size_t)h];
    for (int part = 0; part < parts; part++) {
      const int row0 = i * bq + part * kBwdRows;
      const int rows_valid = max(0, min(kBwdRows, min(N, (i + 1) * bq) - row0));
      if (rows_valid == 0) continue;                  // uniform: the whole workgroup skips
      __syncthreads();                                // previous step fully consumed (and ks, vs written)
      for (int idx = tid; idx < kBwdRows * D; idx += 256) {
        const int r = idx / D, c = idx % D;
        const bool ok = r < rows_valid;
        qs[r * LD + c] = ok ? load_elem(qh, (size_t)(row0 + r) * sin.n + c) : 0.f;
        dos[r * LD + c] = ok ? al * load_elem(doh, (size_t)(row0 + r) * sout.n + c) : 0.f;
      }
      if (tid < kBwdRows) {
        const bool ok = tid < rows_valid;
        rowl[tid] = ok ? lse[(size_t)bh * N + row0 + tid] : 0.f;
        rowd[tid] = ok ? ds_in[(size_t)bh * N + row0 + tid] : 0.f;
      }
      __syncthreads();
      // S^T and dP^T on key tokens 4 ty + a, query rows tx + 16 b
      float sacc[4][4], pacc[4][4];
#pragma unroll
      for (int a = 0; a < 4; a++)
#pragma unroll
        for (int b = 0; b < 4; b++) { sacc[a][b] = 0.f; pacc[a][b] = 0.f; }
      for (int c = 0; c < D; c++) {
        float kv[4], vv[4], qv[4], gv[4];
#pragma unroll
        for (int a = 0; a < 4; a++) { kv[a] = ks[(4 * ty + a) * LD + c]; vv[a] = vs[(4 * ty + a) * LD + c]; }
#pragma unroll
        for (int b = 0; b < 4; b++) { qv[b] = qs[(tx + 16 * b) * LD + c]; gv[b] = dos[(tx + 16 * b) * LD + c]; }
#pragma unroll
        for (int a = 0; a < 4; a++)
#pragma unroll
          for (int b = 0; b < 4; b++) { sacc[a][b] += kv[a] * qv[b]; pacc[a][b] += vv[a] * gv[b]; }
      }
      float pv[4][4];
#pragma unroll
      for (int a = 0; a < 4; a++)
#pragma unroll
        for (int b = 0; b < 4; b++) {
          const int r = tx + 16 * b;
          const bool ok = (4 * ty + a) < valid && r < rows_valid;
          pv[a][b] = ok ? __expf(sacc[a][b] * rscale - rowl[r]) : 0.f;
          ps[r * LP + 4 * ty + a] = pv[a][b];         // P[row][token]
        }
      __syncthreads();
      // dV[token][c] += sum_rows P[row][token] dO^s[row][c]
      for (int r = 0; r < kBwdRows; r++) {
        float pr[4], gv[OC];
#pragma unroll
        for (int a = 0; a < 4; a++) pr[a] = ps[r * LP + 4 * ty + a];
#pragma unroll
        for (int b = 0; b < OC; b++) gv[b] = dos[r * LD + tx + 16 * b];
#pragma unroll
        for (int a = 0; a < 4; a++)
#pragma unroll
          for (int b = 0; b < OC; b++) dvacc[a][b] += pr[a] * gv[b];
      }
      __syncthreads();                                // P fully consumed
#pragma unroll
      for (int a = 0; a < 4; a++)
#pragma unroll
        for (int b = 0; b < 4; b++) {
          const int r = tx + 16 * b;
          ps[r * LP + 4 * ty + a] = pv[a][b] * (pacc[a][b] - rowd[r]);     // dS[row][token]
        }
      __syncthreads();
      // dK'[token][c] += sum_rows dS[row][token] Q[row][c]   (the 1 / sqrt d is applied once at the end)
      for (int r = 0; r < kBwdRows; r++) {
        float sr[4], qv[OC];
#pragma unroll
        for (int a = 0; a < 4; a++) sr[a] = ps[r * LP + 4 * ty + a];
#pragma unroll
        for (int b = 0; b < OC; b++) qv[b] = qs[r * LD + tx + 16 * b];
#pragma unroll
        for (int a = 0; a < 4; a++)
#pragma unroll
          for (int b = 0; b < OC; b++) dkacc[a][b] += sr[a] * qv[b];
      }
    }
  }
  __syncthreads();

  // ---- linear branch: dH = dH_total - sum over the query blocks that selected j of dH_i ----
  const bool all_selected = ksel >= Tn;
  float dhj[MT][MT];
  {
    const float* tot = dh_total + (size_t)bh * D * D;
#pragma unroll
    for (int a = 0; a < MT; a++)
#pragma unroll
      for (int b = 0; b < MT; b++) dhj[a][b] = all_selected ? 0.f : tot[(MT * ty + a) * D + tx + 16 * b];
    float dzj = (tid < D && !all_selected) ? dz_total[(size_t)bh * D + tid] : 0.f;
    if (!all_selected)
      for (int l = l0; l < l1; l++)
        for (int part = 0; part < parts; part++) {
          const size_t slot = ((size_t)bh * Tm + ci[l]) * parts + part;
          const float* src = dh_in + slot * D * D;
#pragma unroll
          for (int a = 0; a < MT; a++)
#pragma unroll
            for (int b = 0; b < MT; b++) dhj[a][b] -= src[(MT * ty + a) * D + tx + 16 * b];
          if (tid < D) dzj -= dz_in[slot * D + tid];
        }
    if (tid < D) dzs[tid] = dzj;
  }
  // K' -> K^phi in place
  for (int idx = tid; idx < kBwdBK * D; idx += 256) {
    const int t = idx / D, c = idx % D;
    float kp = 0.f;
    if (t < valid) kp = __expf(ks[t * LD + c] - k_stats[(size_t)bh * N + t0 + t]);
    ks[t * LD + c] = kp;
  }
#pragma unroll
  for (int a = 0; a < MT; a++)
#pragma unroll
    for (int b = 0; b < MT; b++) dhs[(MT * ty + a) * D + tx + 16 * b] = dhj[a][b];      // dH[c][e]
  __syncthreads();
  // dV[token][e] += sum_c K^phi[token][c] dH[c][e]
  for (int c = 0; c < D; c++) {
    float kp[4], hv[OC];
#pragma unroll
    for (int a = 0; a < 4; a++) kp[a] = ks[(4 * ty + a) * LD + c];
#pragma unroll
    for (int b = 0; b < OC; b++) hv[b] = dhs[c * D + tx + 16 * b];
#pragma unroll
    for (int a = 0; a < 4; a++)
#pragma unroll
      for (int b = 0; b < OC; b++) dvacc[a][b] += kp[a] * hv[b];
  }
  __syncthreads();
#pragma unroll
  for (int a = 0; a < MT; a++)
#pragma unroll
    for (int b = 0; b < MT; b++) dhs[(tx + 16 * b) * D + MT * ty + a] = dhj[a][b];      // dH^T[e][c]
  __syncthreads();
  // dK^phi[token][c] = sum_e V[token][e] dH[c][e] + dZ[c]
  float dkp[4][OC];
#pragma unroll
  for (int a = 0; a < 4; a++)
#pragma unroll
    for (int b = 0; b < OC; b++) dkp[a][b] = dzs[tx + 16 * b];
  for (int e = 0; e < D; e++) {
    float vv[4], hv[OC];
#pragma unroll
    for (int a = 0; a < 4; a++) vv[a] = vs[(4 * ty + a) * LD + e];
#pragma unroll
    for (int b = 0; b < OC; b++) hv[b] = dhs[e * D + tx + 16 * b];
#pragma unroll
    for (int a = 0; a < 4; a++)
#pragma unroll
      for (int b = 0; b < OC; b++) dkp[a][b] += vv[a] * hv[b];
  }
  // back through the softmax, add the sparse part, store; column sums of dK' for the smoothing term
  T* dkh = dk + head_offset(sin, bh, H);
  T* dvh = dv + head_offset(sin, bh, H);
  float csum[OC];
#pragma unroll
  for (int b = 0; b < OC; b++) csum[b] = 0.f;
#pragma unroll
  for (int a = 0; a < 4; a++) {
    const int t = 4 * ty + a;
    float dot = 0.f;
#pragma unroll
    for (int b = 0; b < OC; b++) dot += dkp[a][b] * ks[t * LD + tx + 16 * b];
    dot = row_sum16(dot);
    if (t < valid) {
#pragma unroll
      for (int b = 0; b < OC; b++) {
        const int c = tx + 16 * b;
        const float g = dkacc[a][b] * rscale + ks[t * LD + c] * (dkp[a][b] - dot);
        csum[b] += g;
        store_elem(dkh, (size_t)(t0 + t) * sin.n + c, g);
        store_elem(dvh, (size_t)(t0 + t) * sin.n + c, dvacc[a][b]);
      }
    }
  }
#pragma unroll
  for (int b = 0; b < OC; b++) red[ty * D + tx + 16 * b] = csum[b];
  __syncthreads();
  if (tid < D) {
    float t = 0.f;
    for (int g = 0; g < 16; g++) t += red[g * D + tid];
    colsum[((size_t)bh * Tn + j) * D + tid] = t;
  }
}

// ---------------------------------------------------------------------------------------------
// mean[bh][c] = sum_j colsum[bh][j][c] / N: 1024 / d interleaved subsets of j, combined in a fixed order
__global__ __launch_bounds__(1024) void bwd_colmean_kernel(const float* __restrict__ colsum, float* __restrict__ mean,
                                                           int Tn, int N, int d) {
  __shared__ float part[1024];
  const int bh = blockIdx.x, tid = threadIdx.x, c = tid % d, sub = tid / d, subs = 1024 / d;
  float s = 0.f;
#pragma unroll 4
  for (int j = sub; j < Tn; j += subs) s += colsum[((size_t)bh * Tn + j) * d + c];
  part[tid] = s;
  __syncthreads();
  if (tid < d) {
    float t = 0.f;
    for (int g = 0; g < subs; g++) t += part[g * d + tid];
    mean[(size_t)bh * d + tid] = t / (float)N;
  }
}

// dK = dK' - colmean(dK'): the gradient of K' = K - colmean(K); 8 elements (of one row) per thread
template <typename T>
__global__ __launch_bounds__(256) void bwd_unsmooth_kernel(T* __restrict__ dk, const float* __restrict__ mean, Strides sin,
                                                           int H, int N, int d) {
  const int bh = blockIdx.y;
  const size_t e = ((size_t)blockIdx.x * 256 + threadIdx.x) * 8;
  if (e >= (size_t)N * d) return;
  const int t = (int)(e / d), c = (int)(e % d);
  T* p = dk + head_offset(sin, bh, H) + (size_t)t * sin.n + c;
  const float* m = mean + (size_t)bh * d + c;
  if constexpr (sizeof(T) == 2) {
    bf16x8 x = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
    for (int y = 0; y < 8; y++) x[y] = (__bf16)((float)x[y] - m[y]);
    *reinterpret_cast<bf16x8*>(p) = x;
  } else {
#pragma unroll
    for (int y = 0; y < 8; y++) p[y] -= m[y];
  }
}

// d alpha: per head [H] (sum over batch, query blocks and parts) or per query block [H, T_m] (batch and
// parts).  One workgroup per output; thread t adds the parts t, t + 256, .. and thread 0 the 256 sums.
__global__ __launch_bounds__(256) void bwd_dalpha_kernel(const float* __restrict__ part, float* __restrict__ dalpha, int B,
                                                         int H, int Tm, int parts, int alpha_per_block) {
  __shared__ float red[256];
  const int x = blockIdx.x, tid = threadIdx.x;
  const int h = alpha_per_block ? x / Tm : x;
  const int per_b = alpha_per_block ? parts : Tm * parts;          // consecutive parts of one batch entry
  float s = 0.f;
  for (int y = tid; y < B * per_b; y += 256) {
    const int b = y / per_b, z = y % per_b;
    const size_t first = ((size_t)(b * H + h) * Tm + (alpha_per_block ? x % Tm : 0)) * parts;
    s += part[first + z];
  }
  red[tid] = s;
  __syncthreads();
  if (tid == 0) {
    float t = 0.f;
    for (int y = 0; y < 256; y++) t += red[y];
    dalpha[x] = t;
  }
}

// ---------------------------------------------------------------------------------------------
constexpr size_t bwd_smem_q(int D) { return ((size_t)4 * 64 * (D + 1) + 64 * 65 + D + 64 + 64 + 256) * sizeof(float); }
constexpr size_t bwd_smem_kv(int D) { return ((size_t)4 * 64 * (D + 1) + 64 * 65 + 64 + 64 + D + 16 * D) * sizeof(float); }

// dH_i, dZ_i and d alpha parts: one slot per query block (bf16 tensors) or per 64 query rows (fp32 tensors)
static int bwd_slots_per_block(const Shape& s) { return s.bf16 ? 1 : s.bq / kBwdRows; }

hipError_t launch_bwd_lists(const Shape& s, const BwdArgs& a, hipStream_t stream) {
  // k = 0: every list is empty (the bit rows are all zero)
  bwd_mask_bits_kernel<<<dim3((unsigned)(s.BH * s.Tm)), 64, 0, stream>>>(a.block_idx, a.mask_bits, s.Tn, s.k);
  const dim3 words((unsigned)((s.Tn + 31) / 32), (unsigned)s.BH);
  bwd_col_count_kernel<<<words, 64, 0, stream>>>(a.mask_bits, a.col_cnt, s.Tm, s.Tn);
  bwd_col_scan_kernel<<<dim3((unsigned)s.BH), 256, 0, stream>>>(a.col_cnt, a.col_ptr, s.Tn);
  bwd_col_fill_kernel<<<words, 64, 0, stream>>>(a.mask_bits, a.col_ptr, a.col_idx, s.Tm, s.Tn, s.k);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_bwd_q_f32(const Shape& s, const BwdArgs& a, hipStream_t stream) {
  static OncePerDevice once;
  if (hipError_t e = allow_dynamic_lds(once, (const void*)bwd_q_kernel<float, D>, (int)bwd_smem_q(D)); e != hipSuccess) return e;
  const int parts = s.bq / kBwdRows;
  bwd_q_kernel<float, D><<<dim3((unsigned)((size_t)s.BH * s.Tm * parts)), 256, bwd_smem_q(D), stream>>>(
      (const float*)a.q, (const float*)a.k, (const float*)a.v, (const float*)a.dout, (const float*)a.o_s,
      (const float*)a.o_l, a.lse, a.k_mean, a.k_stats, a.h_total, a.z_total, a.block_idx, a.alpha, (float*)a.dq, a.ds,
      (float*)a.dh, a.dz, a.dalpha_part, s.sin, s.sout, s.H, s.N, s.bq, s.Tm, s.Tn, s.k, s.alpha_per_block ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch_bwd_q(const Shape& s, const BwdArgs& a, hipStream_t stream) {
  if (s.bf16) return launch_bwd_q_bf16(s, a, stream);
  return s.d == 128 ? launch_bwd_q_f32<128>(s, a, stream) : launch_bwd_q_f32<64>(s, a, stream);
}

hipError_t launch_bwd_totals(const Shape& s, const BwdArgs& a, hipStream_t stream) {
  const int D = s.d, count = s.Tm * bwd_slots_per_block(s);
  const dim3 grid_h((unsigned)((D * D + 255) / 256), (unsigned)s.BH), grid_z((unsigned)((D + 255) / 256), (unsigned)s.BH);
  if (s.bf16) bwd_sum_kernel<uint16_t><<<grid_h, 256, 0, stream>>>((const uint16_t*)a.dh, a.dh_total, count, D * D);
  else bwd_sum_kernel<float><<<grid_h, 256, 0, stream>>>((const float*)a.dh, a.dh_total, count, D * D);
  bwd_sum_kernel<float><<<grid_z, 256, 0, stream>>>(a.dz, a.dz_total, count, D);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_bwd_kv_f32(const Shape& s, const BwdArgs& a, hipStream_t stream) {
  static OncePerDevice once;
  if (hipError_t e = allow_dynamic_lds(once, (const void*)bwd_kv_kernel<float, D>, (int)bwd_smem_kv(D)); e != hipSuccess) return e;
  bwd_kv_kernel<float, D><<<dim3((unsigned)((size_t)s.BH * s.Tn)), 256, bwd_smem_kv(D), stream>>>(
      (const float*)a.q, (const float*)a.k, (const float*)a.v, (const float*)a.dout, a.lse, a.ds, a.k_mean, a.k_stats,
      a.col_ptr, a.col_idx, (const float*)a.dh, a.dz, a.dh_total, a.dz_total, a.alpha, (float*)a.dk, (float*)a.dv,
      a.colsum, s.sin, s.sout, s.H, s.N, s.bq, s.Tm, s.Tn, s.k, s.alpha_per_block ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch_bwd_kv(const Shape& s, const BwdArgs& a, hipStream_t stream) {
  if (s.bf16) return launch_bwd_kv_bf16(s, a, stream);
  return s.d == 128 ? launch_bwd_kv_f32<128>(s, a, stream) : launch_bwd_kv_f32<64>(s, a, stream);
}

hipError_t launch_bwd_finish(const Shape& s, const BwdArgs& a, hipStream_t stream) {
  const int D = s.d;
  if (s.smooth) {
    bwd_colmean_kernel<<<dim3((unsigned)s.BH), 1024, 0, stream>>>(a.colsum, a.dk_mean, s.Tn, s.N, D);
    const dim3 grid((unsigned)(((size_t)s.N * D / 8 + 255) / 256), (unsigned)s.BH);
    if (s.bf16) bwd_unsmooth_kernel<uint16_t><<<grid, 256, 0, stream>>>((uint16_t*)a.dk, a.dk_mean, s.sin, s.H, s.N, D);
    else bwd_unsmooth_kernel<float><<<grid, 256, 0, stream>>>((float*)a.dk, a.dk_mean, s.sin, s.H, s.N, D);
  }
  const int n_alpha = s.alpha_per_block ? s.H * s.Tm : s.H;
  bwd_dalpha_kernel<<<dim3((unsigned)n_alpha), 256, 0, stream>>>(a.dalpha_part, a.dalpha, s.B, s.H, s.Tm,
                                                                 bwd_slots_per_block(s), s.alpha_per_block ? 1 : 0);
  return hipGetLastError();
}

}  // namespace sla2
