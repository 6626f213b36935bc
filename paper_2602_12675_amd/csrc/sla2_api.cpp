// Host side of libsla2: argument validation, workspace carve-up, kernel launches.
// Declarations and their contracts are in include/sla2.h.
#include <math.h>
#include <stdint.h>
#include <string.h>

#include <atomic>
#include <vector>

#include "common.h"

namespace sla2 {

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Validate everything that does not need pointers and derive the block counts.
int make_shape(const sla2_params* p, Shape* s) {
  if (!p) return SLA2_EINVAL;
  if (p->B < 1 || p->H < 1 || p->N < 1) return SLA2_EINVAL;
  if (!(p->topk_frac >= 0.0f && p->topk_frac <= 1.0f)) return SLA2_EINVAL;   // also rejects NaN
  if (p->dtype != SLA2_F32 && p->dtype != SLA2_BF16) return SLA2_EINVAL;
  if (p->quant_mode != SLA2_QUANT_NONE && p->quant_mode != SLA2_QUANT_FP8 && p->quant_mode != SLA2_QUANT_INT8 &&
      p->quant_mode != SLA2_QUANT_FP8_V)
    return SLA2_EINVAL;
  if (p->router_w_per_head != 0 && p->router_w_per_head != 1) return SLA2_EINVAL;
  if (p->alpha_per_block != 0 && p->alpha_per_block != 1) return SLA2_EINVAL;
  if (p->flags & ~(SLA2_FLAG_NO_SMOOTH_K | SLA2_FLAG_SAVE_FOR_BACKWARD)) return SLA2_EINVAL;
  if (p->d != 64 && p->d != 128) return SLA2_EUNSUPPORTED;
  if (!((p->block_q == 64 || p->block_q == 128) && p->block_kv == 64)) return SLA2_EUNSUPPORTED;
  if (p->quant_mode != SLA2_QUANT_NONE && p->dtype != SLA2_BF16) return SLA2_EUNSUPPORTED;
  if ((long long)p->B * p->H > 65535) return SLA2_EUNSUPPORTED;
  s->B = p->B; s->H = p->H; s->N = p->N; s->d = p->d; s->bq = p->block_q; s->bk = p->block_kv;
  s->BH = p->B * p->H;
  s->Tm = (p->N + p->block_q - 1) / p->block_q;
  s->Tn = (p->N + p->block_kv - 1) / p->block_kv;
  if (s->Tn > kMaxKeyBlocks) return SLA2_EUNSUPPORTED;
  int k = (int)floor((double)p->topk_frac * (double)s->Tn + 0.5);
  s->k = k < 0 ? 0 : (k > s->Tn ? s->Tn : k);
  s->bf16 = p->dtype == SLA2_BF16;
  {
    const long long esz = s->bf16 ? 2 : 4;
    const long long dflt[3] = {(long long)p->H * p->N * p->d, (long long)p->N * p->d, (long long)p->d};
    Strides* dst[2] = {&s->sin, &s->sout};
    const long long* src[2] = {p->in_stride, p->out_stride};
    for (int x = 0; x < 2; x++) {
      const long long* st = src[x];
      const bool unset = st[0] == 0 && st[1] == 0 && st[2] == 0;
      const long long b = unset ? dflt[0] : st[0], h = unset ? dflt[1] : st[1], n = unset ? dflt[2] : st[2];
      if (b <= 0 || h <= 0 || n <= 0) return SLA2_EINVAL;
      if (n < p->d || n >= (1 << 24)) return SLA2_EUNSUPPORTED;
      if ((b * esz) % 16 || (h * esz) % 16 || (n * esz) % 16) return SLA2_EUNSUPPORTED;
      dst[x]->b = b; dst[x]->h = h; dst[x]->n = (int)n;
    }
  }
  s->quant = (int)p->quant_mode;
  s->smooth = !(p->flags & SLA2_FLAG_NO_SMOOTH_K);
  s->save = (p->flags & SLA2_FLAG_SAVE_FOR_BACKWARD) != 0;
  s->w_per_head = p->router_w_per_head != 0;
  s->alpha_per_block = p->alpha_per_block != 0;
  // Key blocks per kv-precompute workgroup.  That kernel keeps 2 workgroups resident per CU (its
  // d x d accumulator costs registers), 512 on the 256 CUs of an MI355X; one workgroup more than that
  // would wait for a free slot and double the kernel's time, so the head's blocks are cut into the
  // largest number of chunks that still fits in one resident set.
  const int kResident = 512;
  int chunks_max = kResident / s->BH;
  if (chunks_max < 1) chunks_max = 1;
  int bpc = (s->Tn + chunks_max - 1) / chunks_max;
  if (bpc < 1) bpc = 1;
  s->blocks_per_chunk = bpc;
  s->chunks = (s->Tn + bpc - 1) / bpc;
  return SLA2_OK;
}

// scratch of the backward pass, carved out of the `bwd` region of the workspace
struct BwdLayout {
  size_t ds, dh, dz, dh_total, dz_total, colsum, dk_mean, dalpha_part, col_ptr, col_idx, col_cnt, mask_bits, h_i, z_i, lraw, total;
};
static BwdLayout make_bwd_layout(const Shape& s) {
  BwdLayout B;
  size_t off = 0, BH = (size_t)s.BH, d = (size_t)s.d;
  auto take = [&](size_t bytes) { size_t o = off; off = align256(off + bytes); return o; };
  // dH_i, dZ_i, d alpha parts: one slot per query block (bf16 tensors; dH_i as bf16) or per 64 query rows (fp32)
  const size_t slots = BH * s.Tm * (size_t)(s.bf16 ? 1 : s.bq / 64);
  B.ds = take(BH * (size_t)s.N * sizeof(float));
  B.dh = take(slots * d * d * (s.bf16 ? 2 : sizeof(float)));
  B.dz = take(slots * d * sizeof(float));
  B.dh_total = take(BH * d * d * sizeof(float));
  B.dz_total = take(BH * d * sizeof(float));
  B.colsum = take(BH * (size_t)s.Tn * d * sizeof(float));
  B.dk_mean = take(BH * d * sizeof(float));
  B.dalpha_part = take(slots * sizeof(float));
  B.col_ptr = take(BH * (size_t)(s.Tn + 1) * sizeof(int32_t));
  B.col_idx = take(BH * s.Tm * (size_t)(s.k > 0 ? s.k : 1) * sizeof(int32_t));
  B.col_cnt = take(BH * (size_t)s.Tn * sizeof(int32_t));
  B.mask_bits = take(BH * s.Tm * (size_t)((s.Tn + 31) / 32) * sizeof(uint32_t));
  // bf16 tensors: the forward kernel leaves H_i^T (bf16) and Z_i per query block here; L on the raw keys
  B.h_i = take(s.bf16 ? BH * s.Tm * d * d * 2 : 0);
  B.z_i = take(s.bf16 ? BH * s.Tm * d * sizeof(float) : 0);
  B.lraw = take(s.bf16 ? BH * (size_t)s.N * sizeof(float) : 0);
  B.total = off;
  return B;
}
static size_t bwd_scratch_bytes(const Shape& s) { return make_bwd_layout(s).total; }

void make_layout(const Shape& s, sla2_ws_layout* L) {
  size_t off = 0, BH = (size_t)s.BH, d = (size_t)s.d;
  auto take = [&](size_t bytes) { size_t o = off; off = align256(off + bytes); return o; };
  L->q_sum = take(BH * s.Tm * d * sizeof(double));
  L->k_sum = take(BH * s.Tn * d * sizeof(double));
  L->k_mean = take(BH * d * sizeof(double));
  L->router_m = take((size_t)(s.w_per_head ? s.H : 1) * d * d * sizeof(double));
  L->block_idx = take(BH * s.Tm * (size_t)(s.k > 0 ? s.k : 1) * sizeof(int32_t));
  L->h_total = take(BH * d * d * sizeof(float));
  L->z_total = take(BH * d * sizeof(float));
  L->k_stats = take(BH * (size_t)s.N * sizeof(float));
  L->k_phi = take(s.bf16 ? BH * (size_t)s.Tn * s.bk * d * 2 : 0);
  L->z_blocks = take(s.bf16 ? BH * (size_t)s.Tn * d * sizeof(float) : 0);
  L->k_fp8 = take(s.quant ? BH * (size_t)s.Tn * s.bk * d : 0);
  L->k_scale = take(s.quant ? BH * (size_t)s.Tn * sizeof(float) : 0);
  L->v_fp8 = take(s.quant == 3 ? BH * (size_t)s.Tn * s.bk * d : 0);
  L->v_scale = take(s.quant == 3 ? BH * (size_t)s.Tn * sizeof(float) : 0);
  L->partial = take(BH * (size_t)s.chunks * (d * d + d) * sizeof(float));
  const size_t esz = s.bf16 ? 2 : 4;
  L->o_s = take(s.save ? BH * (size_t)s.N * d * esz : 0);
  L->o_l = take(s.save && !s.bf16 ? BH * (size_t)s.N * d * esz : 0);   // bf16 tensors: rebuilt from H_i in the backward pass
  L->lse = take(s.save ? BH * (size_t)s.N * sizeof(float) : 0);
  L->bwd = take(s.save ? bwd_scratch_bytes(s) : 0);
  L->total = off;
}

// bytes from the first to one past the last element a strided [B, H, N, d] view touches
static size_t span_bytes(const Shape& s, const Strides& st) {
  const size_t elems = (size_t)(s.B - 1) * (size_t)st.b + (size_t)(s.H - 1) * (size_t)st.h +
                       (size_t)(s.N - 1) * (size_t)st.n + (size_t)s.d;
  return elems * (s.bf16 ? 2 : 4);
}
static bool misaligned16(const void* p) { return ((uintptr_t)p & 15u) != 0; }

static bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
  uintptr_t x = (uintptr_t)a, y = (uintptr_t)b;
  return x < y + nb && y < x + na;
}

// Two tensors of the same strides whose address ranges interleave (slices of one packed projection,
// [.., N, x, H, d]): they are disjoint when every token period holds each of them in its own stretch.
// With the batch stride a multiple of the token stride, a tensor occupies the offsets
// [r, r + (H - 1) head_stride + d) of every period; the two stretches must not meet (nor wrap).
static bool interleaved_disjoint(const Shape& s, const Strides& st, const void* a, const void* b) {
  const long long esz = s.bf16 ? 2 : 4, period = st.n;
  if (st.h < s.d || (s.B > 1 && st.b % period != 0)) return false;
  const long long extent = (long long)(s.H - 1) * st.h + s.d;
  if (extent > period) return false;
  const long long delta = ((long long)(intptr_t)b - (long long)(intptr_t)a) / esz;
  const long long r = ((delta % period) + period) % period;
  return r >= extent && r <= period - extent;
}

static int check_workspace(const sla2_ws_layout& L, const void* ws, size_t bytes) {
  if (!ws || ((uintptr_t)ws & 255) || bytes < L.total) return SLA2_EWORKSPACE;
  return SLA2_OK;
}

template <class T>
static T* at(void* ws, size_t off) { return (T*)((char*)ws + off); }

// ---- optional per-stage event timing (see sla2_profile_begin in sla2.h) ----
// Calls made while no profile is open only read `active` (atomic): they share no mutable state, so
// the entry points may be used from several threads.  An open profile is single-threaded by contract.
struct Profiler {
  std::atomic<bool> active{false};
  unsigned mask = 0;
  int max_calls = 0, calls = 0, every = 1;          // every-th call is bracketed; max_calls of them
  std::vector<hipEvent_t> pool;                   // created in begin(); two per (call, stage)
  struct Rec { int stage; hipEvent_t a, b; };
  std::vector<Rec> recs;                          // capacity reserved in begin()
  size_t next = 0;
};
static Profiler g_prof;

// Brackets one launch with events when profiling asks for it.
struct StageTimer {
  hipStream_t st; int stage; bool on = false; hipEvent_t a, b;
  StageTimer(int stage_, hipStream_t st_) : st(st_), stage(stage_) {
    Profiler& p = g_prof;
    if (p.active && (p.mask >> stage & 1u) && (p.calls - 1) % p.every == 0 && (p.calls - 1) / p.every < p.max_calls &&
        p.next + 2 <= p.pool.size() &&
        p.recs.size() < p.recs.capacity()) {
      a = p.pool[p.next++]; b = p.pool[p.next++];
      on = hipEventRecord(a, st) == hipSuccess;
    }
  }
  ~StageTimer() {
    if (on && hipEventRecord(b, st) == hipSuccess) g_prof.recs.push_back({stage, a, b});
  }
};
#define SLA2_STAGE(stage, call) ([&]() { StageTimer t_(stage, st); return (call); }())
static void count_call() { if (g_prof.active.load(std::memory_order_acquire)) g_prof.calls++; }

// pool -> colmean -> project -> scores + top-k.  Leaves the index lists in the workspace.
static int run_router(const Shape& s, const sla2_ws_layout& L, const void* q, const void* k, const float* router_w,
                      void* ws, hipStream_t st) {
  double* q_sum = at<double>(ws, L.q_sum);
  double* k_sum = at<double>(ws, L.k_sum);
  double* router_m = at<double>(ws, L.router_m);
  if (SLA2_STAGE(SLA2_STAGE_BLOCK_SUMS, launch_block_sums(s, q, k, router_w, q_sum, k_sum, router_m, st)) !=
      hipSuccess)
    return SLA2_EHIP;
  if (SLA2_STAGE(SLA2_STAGE_TOPK, launch_router_topk(s, q_sum, k_sum, router_m, at<int32_t>(ws, L.block_idx),
                                                     at<double>(ws, L.k_mean), st)) != hipSuccess)
    return SLA2_EHIP;
  return SLA2_OK;
}

}  // namespace sla2

using namespace sla2;

extern "C" {

size_t sla2_workspace_bytes(const sla2_params* params) {
  Shape s; sla2_ws_layout L;
  if (make_shape(params, &s) != SLA2_OK) return 0;
  make_layout(s, &L);
  return L.total;
}

int sla2_workspace_layout(const sla2_params* params, sla2_ws_layout* out) {
  if (!out) return SLA2_EINVAL;
  memset(out, 0, sizeof(*out));
  Shape s;
  int rc = make_shape(params, &s);
  if (rc != SLA2_OK) return rc;
  make_layout(s, out);
  return SLA2_OK;
}

int sla2_num_selected(const sla2_params* params) {
  Shape s;
  int rc = make_shape(params, &s);
  return rc != SLA2_OK ? rc : s.k;
}

int sla2_router(const sla2_params* params, const void* q, const void* k, const float* router_w, int32_t* block_idx,
                void* workspace, size_t workspace_bytes, void* hip_stream) {
  Shape s; sla2_ws_layout L;
  int rc = make_shape(params, &s);
  if (rc != SLA2_OK) return rc;
  if (!q || !k || !router_w || (!block_idx && s.k > 0)) return SLA2_EINVAL;
  if (misaligned16(q) || misaligned16(k)) return SLA2_EINVAL;
  make_layout(s, &L);
  if ((rc = check_workspace(L, workspace, workspace_bytes)) != SLA2_OK) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  count_call();
  if ((rc = run_router(s, L, q, k, router_w, workspace, st)) != SLA2_OK) return rc;
  if (s.k > 0) {
    size_t bytes = (size_t)s.BH * s.Tm * s.k * sizeof(int32_t);
    if (hipMemcpyAsync(block_idx, at<int32_t>(workspace, L.block_idx), bytes, hipMemcpyDeviceToDevice, st) != hipSuccess)
      return SLA2_EHIP;
  }
  return SLA2_OK;
}

int sla2_router_soft(const sla2_params* params, const void* q, const void* k, const float* router_w, float tau,
                     float* mask_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  Shape s; sla2_ws_layout L;
  int rc = make_shape(params, &s);
  if (rc != SLA2_OK) return rc;
  if (!q || !k || !router_w || !mask_out || !(tau > 0.f)) return SLA2_EINVAL;
  if (misaligned16(q) || misaligned16(k)) return SLA2_EINVAL;
  make_layout(s, &L);
  if ((rc = check_workspace(L, workspace, workspace_bytes)) != SLA2_OK) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  count_call();
  if (SLA2_STAGE(SLA2_STAGE_BLOCK_SUMS, launch_block_sums(s, q, k, router_w, at<double>(workspace, L.q_sum),
                                                          at<double>(workspace, L.k_sum),
                                                          at<double>(workspace, L.router_m), st)) != hipSuccess)
    return SLA2_EHIP;
  if (SLA2_STAGE(SLA2_STAGE_TOPK, launch_router_soft(s, at<double>(workspace, L.q_sum), at<double>(workspace, L.k_sum),
                                                     at<double>(workspace, L.router_m), mask_out, (double)tau,
                                                     st)) != hipSuccess)
    return SLA2_EHIP;
  return SLA2_OK;
}

int sla2_forward(const sla2_params* params, const void* q, const void* k, const void* v, const float* router_w,
                 const float* alpha, void* out, int32_t* block_idx_or_null, float* lse_or_null, void* workspace,
                 size_t workspace_bytes, void* hip_stream) {
  Shape s; sla2_ws_layout L;
  int rc = make_shape(params, &s);
  if (rc != SLA2_OK) return rc;
  if (!q || !k || !v || !router_w || !alpha || !out) return SLA2_EINVAL;
  if (misaligned16(q) || misaligned16(k) || misaligned16(v) || misaligned16(out)) return SLA2_EINVAL;
  const size_t in_bytes = span_bytes(s, s.sin), out_bytes = span_bytes(s, s.sout);
  if (overlaps(out, out_bytes, q, in_bytes) || overlaps(out, out_bytes, k, in_bytes) ||
      overlaps(out, out_bytes, v, in_bytes))
    return SLA2_EALIAS;
  make_layout(s, &L);
  if ((rc = check_workspace(L, workspace, workspace_bytes)) != SLA2_OK) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  count_call();
  if ((rc = run_router(s, L, q, k, router_w, workspace, st)) != SLA2_OK) return rc;
  int32_t* idx = at<int32_t>(workspace, L.block_idx);
  if (block_idx_or_null && s.k > 0) {
    size_t bytes = (size_t)s.BH * s.Tm * s.k * sizeof(int32_t);
    if (hipMemcpyAsync(block_idx_or_null, idx, bytes, hipMemcpyDeviceToDevice, st) != hipSuccess) return SLA2_EHIP;
  }
  const double* k_mean = at<double>(workspace, L.k_mean);
  SavedForBackward sv{nullptr, nullptr, nullptr, nullptr, nullptr};
  if (s.save) {
    sv = SavedForBackward{at<void>(workspace, L.o_s), at<void>(workspace, L.o_l), at<float>(workspace, L.lse), nullptr, nullptr};
    if (s.bf16) {
      sv.o_l = nullptr;
      const BwdLayout B = make_bwd_layout(s);
      sv.h_i = (uint16_t*)(at<char>(workspace, L.bwd) + B.h_i);
      sv.z_i = (float*)(at<char>(workspace, L.bwd) + B.z_i);
    }
  }
  float* k_stats = at<float>(workspace, L.k_stats);
  float* h_total = at<float>(workspace, L.h_total);
  float* z_total = at<float>(workspace, L.z_total);
  float* partial = at<float>(workspace, L.partial);
  if (!s.bf16) {
    if (SLA2_STAGE(SLA2_STAGE_KV_STATE, launch_kv_state_f32(s, (const float*)k, (const float*)v, k_mean, k_stats,
                                                            partial, st)) != hipSuccess)
      return SLA2_EHIP;
    if (SLA2_STAGE(SLA2_STAGE_KV_TOTAL, launch_kv_total(s, partial, h_total, z_total, st)) != hipSuccess)
      return SLA2_EHIP;
    if (SLA2_STAGE(SLA2_STAGE_ATTN,
                   launch_attn_f32(s, (const float*)q, (const float*)k, (const float*)v, k_mean, k_stats, h_total,
                                   z_total, idx, alpha, (float*)out, lse_or_null, sv, st)) != hipSuccess)
      return SLA2_EHIP;
    return SLA2_OK;
  }
  uint16_t* k_phi = at<uint16_t>(workspace, L.k_phi);
  float* z_blocks = at<float>(workspace, L.z_blocks);
  uint8_t* k_fp8 = at<uint8_t>(workspace, L.k_fp8);
  float* k_scale = at<float>(workspace, L.k_scale);
  uint8_t* v_fp8 = at<uint8_t>(workspace, L.v_fp8);
  float* v_scale = at<float>(workspace, L.v_scale);
  if (SLA2_STAGE(SLA2_STAGE_KV_STATE,
                 launch_kv_state_bf16(s, (const uint16_t*)k, (const uint16_t*)v, k_mean, k_stats, partial, k_phi,
                                      z_blocks, k_fp8, k_scale, v_fp8, v_scale, st)) != hipSuccess)
    return SLA2_EHIP;
  if (SLA2_STAGE(SLA2_STAGE_KV_TOTAL, launch_kv_total(s, partial, h_total, z_total, st)) != hipSuccess)
    return SLA2_EHIP;
  if (SLA2_STAGE(SLA2_STAGE_ATTN,
                 launch_attn_bf16(s, (const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, k_mean, k_phi,
                                  z_blocks, k_fp8, k_scale, v_fp8, v_scale, h_total, z_total, idx, alpha, (uint16_t*)out,
                                  lse_or_null, sv, st)) != hipSuccess)
    return SLA2_EHIP;
  return SLA2_OK;
}

int sla2_backward(const sla2_params* params, const void* q, const void* k, const void* v, const float* alpha,
                  const void* dout, void* dq, void* dk, void* dv, float* dalpha, void* workspace,
                  size_t workspace_bytes, void* hip_stream) {
  Shape s; sla2_ws_layout L;
  int rc = make_shape(params, &s);
  if (rc != SLA2_OK) return rc;
  if (!s.save) return SLA2_EINVAL;                     // the forward call did not keep what Alg. 3 needs
  if (!q || !k || !v || !alpha || !dout || !dq || !dk || !dv || !dalpha) return SLA2_EINVAL;
  if (misaligned16(q) || misaligned16(k) || misaligned16(v) || misaligned16(dout) || misaligned16(dq) ||
      misaligned16(dk) || misaligned16(dv))
    return SLA2_EINVAL;
  const size_t in_bytes = span_bytes(s, s.sin);
  const void* ins[4] = {q, k, v, dout};
  void* outs[3] = {dq, dk, dv};
  for (void* o : outs)
    for (int x = 0; x < 4; x++)
      if (overlaps(o, in_bytes, ins[x], x == 3 ? span_bytes(s, s.sout) : in_bytes)) return SLA2_EALIAS;
  void* pairs[3][2] = {{dq, dk}, {dq, dv}, {dk, dv}};
  for (auto& pr : pairs)
    if (overlaps(pr[0], in_bytes, pr[1], in_bytes) && !interleaved_disjoint(s, s.sin, pr[0], pr[1])) return SLA2_EALIAS;
  make_layout(s, &L);
  if ((rc = check_workspace(L, workspace, workspace_bytes)) != SLA2_OK) return rc;
  const BwdLayout B = make_bwd_layout(s);
  char* bw = at<char>(workspace, L.bwd);
  BwdArgs a;
  a.q = q; a.k = k; a.v = v; a.dout = dout;
  a.o_s = at<void>(workspace, L.o_s); a.o_l = at<void>(workspace, L.o_l); a.lse = at<float>(workspace, L.lse);
  a.k_mean = at<double>(workspace, L.k_mean);
  a.k_stats = at<float>(workspace, L.k_stats);
  a.h_total = at<float>(workspace, L.h_total); a.z_total = at<float>(workspace, L.z_total);
  a.block_idx = at<int32_t>(workspace, L.block_idx);
  a.alpha = alpha;
  a.dq = dq; a.dk = dk; a.dv = dv; a.dalpha = dalpha;
  a.h_i = (const uint16_t*)(bw + B.h_i); a.z_i = (const float*)(bw + B.z_i); a.lraw = (float*)(bw + B.lraw);
  a.ds = (float*)(bw + B.ds); a.dh = (void*)(bw + B.dh); a.dz = (float*)(bw + B.dz);
  a.dh_total = (float*)(bw + B.dh_total); a.dz_total = (float*)(bw + B.dz_total);
  a.colsum = (float*)(bw + B.colsum); a.dk_mean = (float*)(bw + B.dk_mean);
  a.dalpha_part = (float*)(bw + B.dalpha_part);
  a.col_ptr = (int32_t*)(bw + B.col_ptr); a.col_idx = (int32_t*)(bw + B.col_idx);
  a.mask_bits = (uint32_t*)(bw + B.mask_bits); a.col_cnt = (int32_t*)(bw + B.col_cnt);
  hipStream_t st = (hipStream_t)hip_stream;
  count_call();
  if (SLA2_STAGE(SLA2_STAGE_BWD_LISTS, launch_bwd_lists(s, a, st)) != hipSuccess) return SLA2_EHIP;
  if (SLA2_STAGE(SLA2_STAGE_BWD_Q, launch_bwd_q(s, a, st)) != hipSuccess) return SLA2_EHIP;
  if (SLA2_STAGE(SLA2_STAGE_BWD_REST, launch_bwd_totals(s, a, st)) != hipSuccess) return SLA2_EHIP;
  if (SLA2_STAGE(SLA2_STAGE_BWD_KV, launch_bwd_kv(s, a, st)) != hipSuccess) return SLA2_EHIP;
  if (SLA2_STAGE(SLA2_STAGE_BWD_REST, launch_bwd_finish(s, a, st)) != hipSuccess) return SLA2_EHIP;
  return SLA2_OK;
}

int sla2_dense_forward(const sla2_params* params, const void* q, const void* k, const void* v, void* out,
                       void* hip_stream) {
  Shape s;
  int rc = make_shape(params, &s);
  if (rc != SLA2_OK) return rc;
  if (!q || !k || !v || !out) return SLA2_EINVAL;
  if (!s.bf16) return SLA2_EUNSUPPORTED;
  if (misaligned16(q) || misaligned16(k) || misaligned16(v) || misaligned16(out)) return SLA2_EINVAL;
  const size_t in_bytes = span_bytes(s, s.sin), out_bytes = span_bytes(s, s.sout);
  if (overlaps(out, out_bytes, q, in_bytes) || overlaps(out, out_bytes, k, in_bytes) ||
      overlaps(out, out_bytes, v, in_bytes))
    return SLA2_EALIAS;
  hipStream_t st = (hipStream_t)hip_stream;
  count_call();
  if (SLA2_STAGE(SLA2_STAGE_DENSE, launch_dense_bf16(s, (const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v,
                                                     (uint16_t*)out, st)) != hipSuccess)
    return SLA2_EHIP;
  return SLA2_OK;
}

int sla2_profile_begin(unsigned stage_mask, int max_calls) { return sla2_profile_begin_sampled(stage_mask, max_calls, 1); }

int sla2_profile_begin_sampled(unsigned stage_mask, int max_calls, int every) {
  Profiler& p = g_prof;
  if (p.active || max_calls < 1 || max_calls > 100000 || every < 1 || (stage_mask >> SLA2_STAGE_COUNT)) return SLA2_EINVAL;
  int per_call = __builtin_popcount(stage_mask);
  if (per_call == 0) return SLA2_EINVAL;
  if (stage_mask >> SLA2_STAGE_BWD_REST & 1u) per_call++;   // that stage is bracketed twice per call (totals, finish)
  size_t n = (size_t)2 * per_call * max_calls;
  p.pool.assign(n, nullptr);
  for (size_t i = 0; i < n; i++)
    if (hipEventCreate(&p.pool[i]) != hipSuccess) {
      for (size_t j = 0; j < i; j++) (void)hipEventDestroy(p.pool[j]);
      p.pool.clear();
      return SLA2_EHIP;
    }
  p.recs.clear();
  p.recs.reserve(n / 2);
  p.next = 0; p.calls = 0; p.max_calls = max_calls; p.every = every; p.mask = stage_mask; p.active = true;
  return SLA2_OK;
}

int sla2_profile_end(double* stage_ms, int* stage_launches) {
  Profiler& p = g_prof;
  if (!p.active || !stage_ms || !stage_launches) return SLA2_EINVAL;
  int rc = SLA2_OK;
  for (int i = 0; i < SLA2_STAGE_COUNT; i++) { stage_ms[i] = 0.0; stage_launches[i] = 0; }
  for (const Profiler::Rec& r : p.recs) {
    float ms = 0.f;
    if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) { rc = SLA2_EHIP; continue; }
    stage_ms[r.stage] += ms;
    stage_launches[r.stage]++;
  }
  for (hipEvent_t e : p.pool) (void)hipEventDestroy(e);
  p.pool.clear(); p.recs.clear(); p.active = false;
  return rc;
}

const char* sla2_strerror(int status) {
  switch (status) {
    case SLA2_OK: return "ok";
    case SLA2_EINVAL: return "invalid argument";
    case SLA2_EUNSUPPORTED: return "unsupported shape or mode";
    case SLA2_EWORKSPACE: return "workspace missing, misaligned or too small";
    case SLA2_EALIAS: return "out overlaps an input";
    case SLA2_EHIP: return "kernel launch failed";
    default: return "unknown status";
  }
}

int sla2_version(void) { return 1; }

}  // extern "C"
