// fp32 path of the SLA2 forward pass (Alg. 2 of the paper): plain fp32 FMA kernels with
// LDS-staged tiles, used when q, k, v are stored in fp32.  The data flow is the one of the
// bf16 / FP8 path - per-head totals of h_j, z_j first, then one pass per query block that
// runs the sparse branch over the selected key/value blocks, rebuilds the h_j, z_j of exactly
// those blocks, subtracts them from the totals, and mixes the two branches - so this file
// also serves as the readable statement of that flow.
#include "common.h"

namespace sla2 {

constexpr int kBK = 64;           // key/value block (b_kv)
constexpr int kRowsF32 = 64;      // query rows per workgroup in the fp32 attention kernel

// ---------------------------------------------------------------------------------------------
// kv_state_f32: for a chunk of key blocks of one head
//   k' = k - colmean(K);  stats[token] = lnZ = log sum_c exp(k'_c);
//   K^phi = softmax_d(k');  partial h += (K^phi_j)^T V_j,  partial z += colsum(K^phi_j)
// (Alg. 2: K^phi, h, z).  Tokens past N contribute nothing.
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void kv_state_f32_kernel(const float* __restrict__ k, const float* __restrict__ v,
                                                           const double* __restrict__ k_mean,
                                                           float* __restrict__ k_stats, float* __restrict__ partial,
                                                           Strides sin, int H, int N, int Tn, int chunks,
                                                           int blocks_per_chunk) {
  constexpr int LD = D + 1;       // odd stride: a column of tokens falls into distinct banks
  constexpr int MT = D / 16;      // micro-tile edge: each thread owns MT x MT entries of h
  extern __shared__ float smem[];
  float* ks = smem;                 // [64][LD]  K' tile, then K^phi tile
  float* vs = smem + kBK * LD;      // [64][LD]  V tile
  __shared__ float mu_s[D];
  const int bh = blockIdx.x / chunks, chunk = blockIdx.x % chunks;
  if (threadIdx.x < D) mu_s[threadIdx.x] = (float)k_mean[(size_t)bh * D + threadIdx.x];
  __syncthreads();
  const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
  const float* kh = k + head_offset(sin, bh, H);
  const float* vh = v + head_offset(sin, bh, H);
  const int j0 = chunk * blocks_per_chunk, j1 = min(Tn, j0 + blocks_per_chunk);

  float hacc[MT][MT];
#pragma unroll
  for (int a = 0; a < MT; a++)
#pragma unroll
    for (int b = 0; b < MT; b++) hacc[a][b] = 0.f;
  float zacc = 0.f;

  for (int j = j0; j < j1; j++) {
    const int t0 = j * kBK, valid = min(kBK, N - t0);
    for (int idx = tid; idx < kBK * D; idx += 256) {
      int t = idx / D, c = idx % D;
      bool ok = t < valid;
      ks[t * LD + c] = ok ? kh[(size_t)(t0 + t) * sin.n + c] - mu_s[c] : 0.f;
      vs[t * LD + c] = ok ? vh[(size_t)(t0 + t) * sin.n + c] : 0.f;
    }
    __syncthreads();
    {  // softmax over the channels of each token, 4 threads per token
      const int t = tid / 4, sub = tid % 4;
      float m = -INFINITY;
      for (int c = sub; c < D; c += 4) m = fmaxf(m, ks[t * LD + c]);
      m = fmaxf(m, __shfl_xor(m, 1));
      m = fmaxf(m, __shfl_xor(m, 2));
      float sum = 0.f;
      for (int c = sub; c < D; c += 4) {
        float e = __expf(ks[t * LD + c] - m);
        ks[t * LD + c] = e;
        sum += e;
      }
      sum += __shfl_xor(sum, 1);
      sum += __shfl_xor(sum, 2);
      const float inv = 1.f / sum;
      const bool ok = t < valid;
      for (int c = sub; c < D; c += 4) ks[t * LD + c] = ok ? ks[t * LD + c] * inv : 0.f;
      if (ok && sub == 0) k_stats[(size_t)bh * N + t0 + t] = m + __logf(sum);
    }
    __syncthreads();
    for (int t = 0; t < kBK; t++) {
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
      for (int t = 0; t < kBK; t++) zacc += ks[t * LD + tid];
    __syncthreads();
  }
  float* ph = partial + (size_t)blockIdx.x * (D * D + D);
#pragma unroll
  for (int a = 0; a < MT; a++)
#pragma unroll
    for (int b = 0; b < MT; b++) ph[(MT * ty + a) * D + tx + 16 * b] = hacc[a][b];
  if (tid < D) ph[D * D + tid] = zacc;
}

// Totals over the chunks of a head (Alg. 2's sums of h_j and z_j over all key blocks).  Each workgroup
// owns 64 entries; its 4 thread groups walk the chunks 4 apart and meet in LDS, always in the same
// order, so the totals are the same bits on every run.
__global__ __launch_bounds__(256) void kv_total_kernel(const float* __restrict__ partial, float* __restrict__ h_total,
                                                       float* __restrict__ z_total, int d, int chunks) {
  __shared__ float red[256];
  const int per_head = d * d + d;
  const int bh = blockIdx.y;
  const int e = blockIdx.x * 64 + threadIdx.x % 64, cg = threadIdx.x / 64;
  float s = 0.f;
  if (e < per_head) {
    const float* p = partial + (size_t)bh * chunks * per_head + e;
#pragma unroll 4
    for (int c = cg; c < chunks; c += 4) s += p[(size_t)c * per_head];
  }
  red[threadIdx.x] = s;
  __syncthreads();
  if (cg == 0 && e < per_head) {
    const float tot = (red[threadIdx.x] + red[threadIdx.x + 64]) + (red[threadIdx.x + 128] + red[threadIdx.x + 192]);
    if (e < d * d) h_total[(size_t)bh * d * d + e] = tot;
    else z_total[(size_t)bh * d + (e - d * d)] = tot;
  }
}

hipError_t launch_kv_total(const Shape& s, const float* partial, float* h_total, float* z_total, hipStream_t stream) {
  int per_head = s.d * s.d + s.d;
  kv_total_kernel<<<dim3((unsigned)((per_head + 63) / 64), (unsigned)s.BH), 256, 0, stream>>>(partial, h_total, z_total,
                                                                                             s.d, s.chunks);
  return hipGetLastError();
}

hipError_t launch_kv_state_f32(const Shape& s, const float* k, const float* v, const double* k_mean, float* k_stats,
                               float* partial, hipStream_t stream) {
  dim3 grid((unsigned)(s.BH * s.chunks));
  const size_t smem = (size_t)2 * kBK * (s.d + 1) * sizeof(float);
  static OncePerDevice once;
  if (hipError_t e0 = allow_dynamic_lds(once, (const void*)kv_state_f32_kernel<128>, 2 * kBK * 129 * (int)sizeof(float)); e0 != hipSuccess) return e0;
  if (s.d == 128)
    kv_state_f32_kernel<128><<<grid, 256, smem, stream>>>(k, v, k_mean, k_stats, partial, s.sin, s.H, s.N, s.Tn, s.chunks,
                                                          s.blocks_per_chunk);
  else
    kv_state_f32_kernel<64><<<grid, 256, smem, stream>>>(k, v, k_mean, k_stats, partial, s.sin, s.H, s.N, s.Tn, s.chunks,
                                                         s.blocks_per_chunk);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// attn_f32: one workgroup per 64 query rows of query block i.
//   sparse branch  : for j in sel(i), ascending: S = Q_i K'_j^T / sqrt(d), online softmax, O += P V_j
//   linear branch  : H_i = H_total - sum_{j in sel(i)} h_j (h_j rebuilt from the staged tiles and the
//                    per-token log-partition lnZ), Z_i likewise; O_l = Q^phi H_i / (Q^phi Z_i)
//   mix            : out = alpha O_s / l + (1 - alpha) O_l                                   (Eq. 13)
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void attn_f32_kernel(const float* __restrict__ q, const float* __restrict__ k,
                                                       const float* __restrict__ v, const double* __restrict__ k_mean,
                                                       const float* __restrict__ k_stats,
                                                       const float* __restrict__ h_total,
                                                       const float* __restrict__ z_total,
                                                       const int32_t* __restrict__ block_idx,
                                                       const float* __restrict__ alpha, float* __restrict__ out,
                                                       float* __restrict__ lse, float* __restrict__ o_s_save,
                                                       float* __restrict__ o_l_save, float* __restrict__ lse_save,
                                                       Strides sin, Strides sout, int H, int N, int bq, int Tm, int Tn,
                                                       int ksel, int alpha_per_block) {
  constexpr int LD = D + 1;
  constexpr int LP = kBK + 1;
  constexpr int MT = D / 16;       // h micro-tile edge
  constexpr int OC = D / 16;       // output columns per thread
  extern __shared__ float smem[];
  float* qs = smem;                       // [64][LD]  Q rows, later Q^phi
  float* ks = qs + kRowsF32 * LD;         // [64][LD]  K' tile, then K^phi tile
  float* vs = ks + kBK * LD;              // [64][LD]  V tile
  float* ps = vs + kBK * LD;              // [64][LP]  P tile
  float* zs = ps + kRowsF32 * LP;         // [D]       Z_i
  float* hs = ks;                         // [D][D]    H_i in the epilogue (covers ks and vs)

  const int parts = bq / kRowsF32;
  int bid = blockIdx.x;
  const int part = bid % parts; bid /= parts;
  const int i = bid % Tm;
  const int bh = bid / Tm;
  const int h = bh % H;
  const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
  const int row0 = i * bq + part * kRowsF32;          // first query row of this workgroup
  const int rows_valid = max(0, min(kRowsF32, min(N, (i + 1) * bq) - row0));
  const float* qh = q + head_offset(sin, bh, H);
  const float* kh = k + head_offset(sin, bh, H);
  const float* vh = v + head_offset(sin, bh, H);
  const int32_t* sel = block_idx + ((size_t)bh * Tm + i) * ksel;
  const float rscale = rsqrtf((float)D);
  if (rows_valid == 0) return;                        // second half of a short last query block

  for (int idx = tid; idx < kRowsF32 * D; idx += 256) {
    int r = idx / D, c = idx % D;
    qs[r * LD + c] = r < rows_valid ? qh[(size_t)(row0 + r) * sin.n + c] : 0.f;
  }

  float m_run[4], l_run[4], oacc[4][OC], hacc[MT][MT];
#pragma unroll
  for (int a = 0; a < 4; a++) {
    m_run[a] = -INFINITY; l_run[a] = 0.f;
#pragma unroll
    for (int b = 0; b < OC; b++) oacc[a][b] = 0.f;
  }
#pragma unroll
  for (int a = 0; a < MT; a++)
#pragma unroll
    for (int b = 0; b < MT; b++) hacc[a][b] = 0.f;
  float zacc = 0.f;

  for (int s = 0; s < ksel; s++) {
    const int j = sel[s];
    const int t0 = j * kBK, valid = min(kBK, N - t0);
    __syncthreads();                                  // previous tile fully consumed (and qs written)
    for (int idx = tid; idx < kBK * D; idx += 256) {
      int t = idx / D, c = idx % D;
      bool ok = t < valid;
      ks[t * LD + c] = ok ? kh[(size_t)(t0 + t) * sin.n + c] - (float)k_mean[(size_t)bh * D + c] : 0.f;
      vs[t * LD + c] = ok ? vh[(size_t)(t0 + t) * sin.n + c] : 0.f;
    }
    __syncthreads();
    // S = Q K'^T / sqrt(d): rows 4 ty + a, key tokens tx + 16 b
    float sacc[4][4];
#pragma unroll
    for (int a = 0; a < 4; a++)
#pragma unroll
      for (int b = 0; b < 4; b++) sacc[a][b] = 0.f;
    for (int c = 0; c < D; c++) {
      float qv[4], kv[4];
#pragma unroll
      for (int a = 0; a < 4; a++) qv[a] = qs[(4 * ty + a) * LD + c];
#pragma unroll
      for (int b = 0; b < 4; b++) kv[b] = ks[(tx + 16 * b) * LD + c];
#pragma unroll
      for (int a = 0; a < 4; a++)
#pragma unroll
        for (int b = 0; b < 4; b++) sacc[a][b] += qv[a] * kv[b];
    }
    float corr[4];
#pragma unroll
    for (int a = 0; a < 4; a++) {
      float mx = -INFINITY;
#pragma unroll
      for (int b = 0; b < 4; b++) {
        sacc[a][b] = (tx + 16 * b) < valid ? sacc[a][b] * rscale : -INFINITY;
        mx = fmaxf(mx, sacc[a][b]);
      }
#pragma unroll
      for (int o = 1; o < 16; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
      const float m_new = fmaxf(m_run[a], mx);        // finite: every block holds at least one token
      float rs = 0.f;
#pragma unroll
      for (int b = 0; b < 4; b++) {
        float p = __expf(sacc[a][b] - m_new);
        ps[(4 * ty + a) * LP + tx + 16 * b] = p;
        rs += p;
      }
#pragma unroll
      for (int o = 1; o < 16; o <<= 1) rs += __shfl_xor(rs, o);
      corr[a] = __expf(m_run[a] - m_new);             // exp(-inf) = 0 on the first block
      l_run[a] = l_run[a] * corr[a] + rs;
      m_run[a] = m_new;
    }
    __syncthreads();                                  // ps complete; ks no longer read as K'
    // K' -> K^phi in place, from the per-token statistics
    for (int idx = tid; idx < kBK * D; idx += 256) {
      int t = idx / D, c = idx % D;
      float kp = 0.f;
      if (t < valid) kp = __expf(ks[t * LD + c] - k_stats[(size_t)bh * N + t0 + t]);
      ks[t * LD + c] = kp;
    }
    // O = diag(corr) O + P V
#pragma unroll
    for (int a = 0; a < 4; a++)
#pragma unroll
      for (int b = 0; b < OC; b++) oacc[a][b] *= corr[a];
    for (int t = 0; t < kBK; t++) {
      float pv[4], vv[OC];
#pragma unroll
      for (int a = 0; a < 4; a++) pv[a] = ps[(4 * ty + a) * LP + t];
#pragma unroll
      for (int b = 0; b < OC; b++) vv[b] = vs[t * LD + tx + 16 * b];
#pragma unroll
      for (int a = 0; a < 4; a++)
#pragma unroll
        for (int b = 0; b < OC; b++) oacc[a][b] += pv[a] * vv[b];
    }
    __syncthreads();                                  // K^phi complete
    for (int t = 0; t < kBK; t++) {
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
      for (int t = 0; t < kBK; t++) zacc += ks[t * LD + tid];
  }
  __syncthreads();

  // ---- linear branch ----
  const bool all_selected = ksel >= Tn;               // nothing left for the linear branch: O_l = 0
  const float* ht = h_total + (size_t)bh * D * D;
#pragma unroll
  for (int a = 0; a < MT; a++)
#pragma unroll
    for (int b = 0; b < MT; b++) {
      int c = MT * ty + a, e = tx + 16 * b;
      hs[c * D + e] = ht[c * D + e] - hacc[a][b];
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
      float e = __expf(qs[r * LD + c] - m);
      qs[r * LD + c] = e;
      sum += e;
    }
    sum += __shfl_xor(sum, 1);
    sum += __shfl_xor(sum, 2);
    const float inv = 1.f / sum;
    for (int c = sub; c < D; c += 4) qs[r * LD + c] *= inv;
  }
  __syncthreads();
  float lacc[4][OC], den[4];
#pragma unroll
  for (int a = 0; a < 4; a++) {
    den[a] = 0.f;
#pragma unroll
    for (int b = 0; b < OC; b++) lacc[a][b] = 0.f;
  }
  for (int c = 0; c < D; c++) {
    float qv[4], hv[OC];
    const float zc = zs[c];
#pragma unroll
    for (int a = 0; a < 4; a++) qv[a] = qs[(4 * ty + a) * LD + c];
#pragma unroll
    for (int b = 0; b < OC; b++) hv[b] = hs[c * D + tx + 16 * b];
#pragma unroll
    for (int a = 0; a < 4; a++) {
      den[a] += qv[a] * zc;
#pragma unroll
      for (int b = 0; b < OC; b++) lacc[a][b] += qv[a] * hv[b];
    }
  }
  // ---- mix and store ----
  const float al = alpha[alpha_per_block ? (size_t)h * Tm + i : (size_t)h];
#pragma unroll
  for (int a = 0; a < 4; a++) {
    const int r = 4 * ty + a;
    if (r >= rows_valid) continue;
    const float inv_l = l_run[a] > 0.f ? 1.f / l_run[a] : 0.f;
    const float inv_den = all_selected ? 0.f : 1.f / den[a];
    float* o = out + head_offset(sout, bh, H) + (size_t)(row0 + r) * sout.n;
#pragma unroll
    for (int b = 0; b < OC; b++) o[tx + 16 * b] = al * oacc[a][b] * inv_l + (1.f - al) * lacc[a][b] * inv_den;
    const float L = l_run[a] > 0.f ? m_run[a] + __logf(l_run[a]) : -INFINITY;
    if (lse && tx == 0) lse[(size_t)bh * N + row0 + r] = L;
    if (o_s_save) {                                   // the two branches and L, kept for the backward pass
      const size_t at = ((size_t)bh * N + row0 + r) * D;
#pragma unroll
      for (int b = 0; b < OC; b++) {
        o_s_save[at + tx + 16 * b] = oacc[a][b] * inv_l;
        o_l_save[at + tx + 16 * b] = lacc[a][b] * inv_den;
      }
      if (tx == 0) lse_save[(size_t)bh * N + row0 + r] = L;
    }
  }
}

template <int D>
static hipError_t launch_attn_f32_t(const Shape& s, const float* q, const float* k, const float* v,
                                    const double* k_mean, const float* k_stats, const float* h_total,
                                    const float* z_total, const int32_t* block_idx, const float* alpha, float* out,
                                    float* lse, const SavedForBackward& sv, hipStream_t stream) {
  size_t smem = ((size_t)3 * 64 * (D + 1) + 64 * 65 + D) * sizeof(float);
  static OncePerDevice once;
  if (hipError_t e = allow_dynamic_lds(once, (const void*)attn_f32_kernel<D>, (int)smem); e != hipSuccess) return e;
  dim3 grid((unsigned)((size_t)s.BH * s.Tm * (s.bq / kRowsF32)));
  attn_f32_kernel<D><<<grid, 256, smem, stream>>>(q, k, v, k_mean, k_stats, h_total, z_total, block_idx, alpha, out,
                                                  lse, (float*)sv.o_s, (float*)sv.o_l, sv.lse, s.sin, s.sout, s.H, s.N,
                                                  s.bq, s.Tm, s.Tn, s.k,
                                                  s.alpha_per_block ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch_attn_f32(const Shape& s, const float* q, const float* k, const float* v, const double* k_mean,
                           const float* k_stats, const float* h_total, const float* z_total, const int32_t* block_idx,
                           const float* alpha, float* out, float* lse, const SavedForBackward& sv,
                           hipStream_t stream) {
  if (s.d == 128)
    return launch_attn_f32_t<128>(s, q, k, v, k_mean, k_stats, h_total, z_total, block_idx, alpha, out, lse, sv, stream);
  return launch_attn_f32_t<64>(s, q, k, v, k_mean, k_stats, h_total, z_total, block_idx, alpha, out, lse, sv, stream);
}

}  // namespace sla2
