// Host side of the S2O C ABI (declared in include/s2o.h): argument validation, size
// queries and kernel launches.  Nothing here allocates device memory or synchronises.
#include <math.h>
#include <string.h>

#include "../../include/s2o.h"

#include <stdlib.h>
#include "s2o_internal.h"

namespace {

thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e) {
  g_last_hip_error = (int)e;
  return S2O_EHIP;
}

struct Shape {
  int Z, H, Hkv, L, D, S, N, nc;
  int64_t qs[3], ks[3], vs[3], os[3];
};

bool fill_strides(const int64_t in[3], int64_t out[3], int heads, int L, int D) {
  if (in[0] == 0 && in[1] == 0 && in[2] == 0) {
    out[2] = D;
    out[1] = (int64_t)L * D;
    out[0] = (int64_t)heads * L * D;
    return true;
  }
  for (int i = 0; i < 3; ++i) {
    if (in[i] < 0 || (in[i] % 8) != 0) return false;   // 16-byte aligned rows
    if (i == 2 && in[i] > (1 << 24)) return false;     // row stride in bytes must fit 32 bits
    out[i] = in[i];
  }
  return out[2] >= D;
}

int check_params(const s2o_params* p, Shape* s, bool for_plan = false) {
  if (!p) return S2O_EINVAL;
  if (p->struct_size != (int32_t)sizeof(s2o_params)) return S2O_EINVAL;
  if (p->batch <= 0 || p->q_heads <= 0 || p->kv_heads <= 0 || p->seq_len <= 0 || p->seg_len <= 0)
    return S2O_EINVAL;
  if (p->q_heads % p->kv_heads != 0) return S2O_EINVAL;
  if (p->seq_len % p->seg_len != 0) return S2O_EINVAL;
  if (p->use_q_perm != 0 && p->use_q_perm != 1) return S2O_EINVAL;
  if (p->stop_mode < 0 || p->stop_mode > 2) return S2O_EINVAL;
  if (p->max_prefix_tiles < 0) return S2O_EINVAL;
  if (p->non_causal != 0 && p->non_causal != 1) return S2O_EINVAL;
  if (!(p->softmax_scale >= 0.f) || isinf(p->softmax_scale)) return S2O_EINVAL;
  if (p->head_dim != 128) return S2O_EUNSUPPORTED;
  if ((p->block_m != 64 && p->block_m != 128) || p->block_n != 64) return S2O_EUNSUPPORTED;
  if (p->seg_len % p->block_m != 0) return S2O_EUNSUPPORTED;
  if (for_plan && p->seg_len > 8192) return S2O_EUNSUPPORTED;   // a segment's query scores are sorted in LDS
  if (for_plan && p->seq_len > (1 << 20)) return S2O_EUNSUPPORTED;   // a row's sample (L/64 scores) is sorted in LDS
  if ((int64_t)p->batch * p->q_heads * (p->seq_len / p->seg_len) > (1 << 24)) return S2O_EUNSUPPORTED;
  s->Z = p->batch; s->H = p->q_heads; s->Hkv = p->kv_heads; s->L = p->seq_len;
  s->D = p->head_dim; s->S = p->seg_len; s->N = p->seq_len / p->seg_len; s->nc = p->non_causal;
  if (!fill_strides(p->q_stride, s->qs, s->H, s->L, s->D)) return S2O_EINVAL;
  if (!fill_strides(p->k_stride, s->ks, s->Hkv, s->L, s->D)) return S2O_EINVAL;
  if (!fill_strides(p->v_stride, s->vs, s->Hkv, s->L, s->D)) return S2O_EINVAL;
  if (!fill_strides(p->o_stride, s->os, s->H, s->L, s->D)) return S2O_EINVAL;
  // the prefix walk addresses a K/V row as a 32-bit byte offset from its head (24-bit multiply)
  for (const int64_t* st : {s->ks, s->vs}) {
    const int64_t row_bytes = st[2] * 2;
    if (row_bytes >= (1 << 24) || (int64_t)(s->L - 1) * row_bytes + 256 > 0xffffffffll) return S2O_EUNSUPPORTED;
  }
  if (s->L > (1 << 24)) return S2O_EUNSUPPORTED;
  return S2O_OK;
}

bool misaligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) != 0; }

// s2o_plan and s2o_plan_static: the same validation and launches; the second takes the
// library's built-in scratch array (looked up per device, nothing allocated).
int plan_call(const void* Q, const void* K, const s2o_params* params, const s2o_plan_out* out, void* scratch,
              size_t scratch_bytes, bool built_in, void* stream) {
  Shape s;
  const int rc = check_params(params, &s, true);
  if (rc != S2O_OK) return rc;
  if (!Q || !K || !out || !out->q_perm) return S2O_EINVAL;
  if ((s.N > 1 || s.nc) && !out->kv_perm) return S2O_EINVAL;
  if (misaligned(Q, 16) || misaligned(K, 16) || misaligned(out->q_perm, 16) ||
      misaligned(out->kv_perm, 16) || misaligned(out->s_k, 16) || misaligned(out->status, 4))
    return S2O_EINVAL;
  const size_t need = s2o::plan_scratch_bytes(s.Z, s.H, s.Hkv, s.L, s.S, s.nc);
  if (built_in) {
    if (need > s2o::kStaticPlanScratchBytes) return S2O_ESCRATCH;   // before any HIP call
    const hipError_t e = s2o::static_plan_scratch(&scratch);
    if (e != hipSuccess) return hip_fail(e);
    scratch_bytes = s2o::kStaticPlanScratchBytes;
  }
  if (!scratch || misaligned(scratch, 256) || scratch_bytes < need) return S2O_ESCRATCH;

  s2o::PlanArgs a;
  memset(&a, 0, sizeof(a));
  a.Q = (const uint16_t*)Q; a.K = (const uint16_t*)K;
  a.q_perm = out->q_perm; a.kv_perm = out->kv_perm;
  a.s_q = out->s_q; a.s_k = out->s_k; a.q_mean = out->q_mean; a.k_guide = out->k_guide;
  a.status = out->status;
  a.Z = s.Z; a.H = s.H; a.Hkv = s.Hkv; a.L = s.L; a.S = s.S; a.N = s.N;
  a.non_causal = s.nc;
  for (int i = 0; i < 3; ++i) { a.qs[i] = s.qs[i]; a.ks[i] = s.ks[i]; }
  a.scratch = scratch; a.scratch_bytes = scratch_bytes;
  const hipError_t e = s2o::launch_plan(a, (hipStream_t)stream);
  return e == hipSuccess ? S2O_OK : hip_fail(e);
}

}  // namespace

extern "C" {

int s2o_version(void) { return S2O_VERSION; }

const char* s2o_strerror(int code) {
  switch (code) {
    case S2O_OK: return "ok";
    case S2O_EINVAL: return "invalid argument";
    case S2O_EUNSUPPORTED: return "unsupported configuration (need D=128, B_M in {64,128}, B_N=64, S%B_M==0; s2o_plan: S<=8192; no own-segment pass when non_causal)";
    case S2O_ESCRATCH: return "scratch buffer missing, misaligned or too small (s2o_plan_static: the configuration needs more than the built-in S2O_STATIC_SCRATCH_BYTES)";
    case S2O_EHIP: return "HIP runtime error (see s2o_last_hip_error)";
    default: return "unknown error code";
  }
}

int s2o_last_hip_error(void) { return g_last_hip_error; }

int s2o_plan_sizes(const s2o_params* params, size_t* q_perm_bytes, size_t* kv_perm_bytes,
                   size_t* s_q_bytes, size_t* s_k_bytes, size_t* q_mean_bytes,
                   size_t* k_guide_bytes, size_t* scratch_bytes) {
  Shape s;
  const int rc = check_params(params, &s, true);
  if (rc != S2O_OK) return rc;
  const size_t zh = (size_t)s.Z * s.H;
  const size_t P = (size_t)s2o::kv_rows_total(s.N, s.S, s.L, s.nc);
  if (q_perm_bytes) *q_perm_bytes = zh * s.L * 4;
  if (kv_perm_bytes) *kv_perm_bytes = zh * P * 4;
  if (s_q_bytes) *s_q_bytes = zh * s.L * 4;
  if (s_k_bytes) *s_k_bytes = zh * P * 4;
  if (q_mean_bytes) *q_mean_bytes = zh * s.N * s.D * 4;
  if (k_guide_bytes) *k_guide_bytes = (size_t)s.Z * s.Hkv * s.D * 4;
  if (scratch_bytes) *scratch_bytes = s2o::plan_scratch_bytes(s.Z, s.H, s.Hkv, s.L, s.S, s.nc);
  return S2O_OK;
}

int s2o_plan(const void* Q, const void* K, const s2o_params* params, const s2o_plan_out* out,
             void* scratch, size_t scratch_bytes, void* stream) {
  return plan_call(Q, K, params, out, scratch, scratch_bytes, false, stream);
}

int s2o_plan_static(const void* Q, const void* K, const s2o_params* params, const s2o_plan_out* out,
                    void* stream) {
  return plan_call(Q, K, params, out, nullptr, 0, true, stream);
}

int s2o_attention_sizes(const s2o_params* params, size_t* counts_bytes, size_t* scratch_bytes) {
  Shape s;
  const int rc = check_params(params, &s);
  if (rc != S2O_OK) return rc;
  if (counts_bytes) *counts_bytes = (size_t)s.Z * s.H * (s.L / params->block_m) * 4;
  if (scratch_bytes) *scratch_bytes = s.nc ? 0 : s2o::attention_state_bytes(s.Z, s.H, s.L);
  return S2O_OK;
}

namespace {
// passes: 1 = own-segment window into the state buffers (Alg. 2), 2 = prefix walk from them
// (Alg. 3), 3 = both; 0 = both in one fused launch without state buffers.
int attention_call(int passes, const void* Q, const void* K, const void* V, const s2o_params* params,
                   const int32_t* q_perm, const int32_t* kv_perm, float tau, void* O,
                   int32_t* computed, int32_t* skipped, void* scratch, size_t scratch_bytes,
                   void* stream) {
  Shape s;
  const int rc = check_params(params, &s);
  if (rc != S2O_OK) return rc;
  if (s.nc) {                               // no own-segment pass and no state: the walk is everything
    if (passes == 1) return S2O_EUNSUPPORTED;
    passes = 2;
  }
  const bool walk = passes != 1;            // the prefix walk is part of this call
  if (!Q || !K || !V) return S2O_EINVAL;
  if (misaligned(Q, 16) || misaligned(K, 16) || misaligned(V, 16)) return S2O_EINVAL;
  if (walk) {
    if (!O || misaligned(O, 16)) return S2O_EINVAL;
    if (params->use_q_perm && !q_perm) return S2O_EINVAL;
    // causal: the prefix rows are needed as soon as a prefix exists; non-causal: NULL means
    // "all keys in storage order" (contiguous dense attention, App. A kernel A)
    if (!s.nc && s.N > 1 && !kv_perm) return S2O_EINVAL;
    if (kv_perm && misaligned(kv_perm, 16)) return S2O_EINVAL;
    if (tau != tau) return S2O_EINVAL;
    if (s.nc && isinf(tau)) return S2O_EINVAL;   // the first tile's test would be inf * 0
  }
  if (passes != 0 && !s.nc &&
      (!scratch || misaligned(scratch, 256) || scratch_bytes < s2o::attention_state_bytes(s.Z, s.H, s.L)))
    return S2O_ESCRATCH;

  s2o::AttnArgs a;
  memset(&a, 0, sizeof(a));
  a.passes = passes;
  a.Q = (const uint16_t*)Q; a.K = (const uint16_t*)K; a.V = (const uint16_t*)V;
  a.O = (uint16_t*)O;
  a.q_perm = q_perm; a.kv_perm = kv_perm; a.computed = computed; a.skipped = skipped;
  a.Z = s.Z; a.H = s.H; a.Hkv = s.Hkv; a.L = s.L; a.S = s.S; a.N = s.N;
  a.BM = params->block_m;
  if (passes != 0 && !s.nc) {
    const size_t rows = (size_t)s.Z * s.H * s.L;
    a.st_acc = (float*)scratch;
    a.st_l = a.st_acc + rows * s.D;
    a.st_m = a.st_l + rows;
  }
  a.use_q_perm = params->use_q_perm; a.stop_mode = params->stop_mode;
  a.max_tiles = params->max_prefix_tiles;
  a.non_causal = s.nc;
  a.tau = tau;
  const float scale = params->softmax_scale > 0.f ? params->softmax_scale : 1.0f / sqrtf((float)s.D);
  a.scale_log2e = scale * 1.4426950408889634f;
  for (int i = 0; i < 3; ++i) {
    a.qs[i] = s.qs[i]; a.ks[i] = s.ks[i]; a.vs[i] = s.vs[i]; a.os[i] = s.os[i];
  }
  if (walk) {
    // debug switch: check the maps' ranges on the device before they are used
    const char* v = getenv("S2O_VALIDATE_MAPS");
    if (v && v[0] && v[0] != '0') {
      int bits = 0;
      const hipError_t ve = s2o::validate_maps(a, (hipStream_t)stream, &bits);
      if (ve != hipSuccess) return hip_fail(ve);
      if (bits) return S2O_EINVAL;
    }
  }
  const hipError_t e = s2o::launch_attention(a, (hipStream_t)stream);
  return e == hipSuccess ? S2O_OK : hip_fail(e);
}
}  // namespace

int s2o_attention(const void* Q, const void* K, const void* V, const s2o_params* params,
                  const int32_t* q_perm, const int32_t* kv_perm, float tau, void* O,
                  int32_t* computed, int32_t* skipped, void* scratch, size_t scratch_bytes,
                  void* stream) {
  return attention_call(scratch ? 3 : 0, Q, K, V, params, q_perm, kv_perm, tau, O, computed, skipped,
                        scratch, scratch_bytes, stream);
}

int s2o_attention_local(const void* Q, const void* K, const void* V, const s2o_params* params,
                        void* scratch, size_t scratch_bytes, void* stream) {
  return attention_call(1, Q, K, V, params, nullptr, nullptr, 0.f, nullptr, nullptr, nullptr, scratch,
                        scratch_bytes, stream);
}

int s2o_attention_prefix(const void* Q, const void* K, const void* V, const s2o_params* params,
                         const int32_t* q_perm, const int32_t* kv_perm, float tau, void* O,
                         int32_t* computed, int32_t* skipped, const void* scratch, size_t scratch_bytes,
                         void* stream) {
  return attention_call(2, Q, K, V, params, q_perm, kv_perm, tau, O, computed, skipped,
                        const_cast<void*>(scratch), scratch_bytes, stream);
}

}  // extern "C"
