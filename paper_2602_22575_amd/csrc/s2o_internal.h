// Internal declarations shared by the host API and the gfx950 kernels of the S2O library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

namespace s2o {

// Packed start of prefix row n (n >= 1) inside one head's KV_perm / s_K array.
__host__ __device__ inline int64_t kv_row_offset(int64_t n, int64_t S) { return S * n * (n - 1) / 2; }

// Rows of KV_perm / s_K for one head.  Causal (the paper's setting): row n ranks the n*S
// tokens before segment n and the rows are packed.  Without causality (params.non_causal,
// the setting of the paper's non-causal decomposition and top-k comparisons) every row
// ranks all L tokens.
__host__ __device__ inline int64_t kv_row_len(int64_t n, int64_t S, int64_t L, int nc) { return nc ? L : n * S; }
__host__ __device__ inline int64_t kv_row_start(int64_t n, int64_t S, int64_t L, int nc) {
  return nc ? n * L : kv_row_offset(n, S);
}
__host__ __device__ inline int64_t kv_rows_total(int64_t N, int64_t S, int64_t L, int nc) {
  return nc ? N * L : kv_row_offset(N, S);
}

// Runs `setup` (kernel attributes such as the dynamic LDS limit are per device) once per
// device, before the first launch there; other host threads wait until it is done.  A failed
// setup is retried by the next call.
template <class F>
inline hipError_t once_per_device(std::mutex& mu, uint64_t& done, F setup) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = 1ull << (dev & 63);
  std::lock_guard<std::mutex> lock(mu);
  if (done & bit) return hipSuccess;
  e = setup();
  if (e == hipSuccess) done |= bit;
  return e;
}

struct AttnArgs {
  const uint16_t* Q;
  const uint16_t* K;
  const uint16_t* V;
  uint16_t* O;
  const int32_t* q_perm;
  const int32_t* kv_perm;
  int32_t* computed;
  int32_t* skipped;
  int passes;     // 0: one fused launch; bit 0: Alg. 2 into the state buffers; bit 1: Alg. 3 from them
  float* st_acc;  // state buffers: acc [Z*H*L][128] (four 128-byte lines per row, see attn_tile.h), then l and m [Z*H*L]
  float* st_l;
  float* st_m;
  int Z, H, Hkv, L, S, N;
  int BM;  // query tile rows (64 or 128); the key tile is 64 tokens
  int use_q_perm, stop_mode;
  int non_causal; // every query attends every key: no own-segment pass, rows of L ranked keys
  int max_tiles;  // > 0: a query tile visits at most this many prefix tiles
  float tau;
  float scale_log2e;  // softmax_scale * log2(e): logits are kept in base-2 units
  int64_t qs[3], ks[3], vs[3], os[3];
};

struct PlanArgs {
  const uint16_t* Q;
  const uint16_t* K;
  int32_t* q_perm;
  int32_t* kv_perm;
  float* s_q;
  float* s_k;
  float* q_mean;
  float* k_guide;
  int32_t* status;   // optional: receives the S2O_PLAN_* bits (0 = every invariant held)
  int Z, H, Hkv, L, S, N;
  int non_causal;
  int64_t qs[3], ks[3];
  void* scratch;
  size_t scratch_bytes;
};

size_t plan_scratch_bytes(int Z, int H, int Hkv, int L, int S, int non_causal);
// Size of the library's built-in plan scratch (S2O_STATIC_SCRATCH_BYTES of the C header) and its
// device address on the current GPU.
constexpr size_t kStaticPlanScratchBytes = (size_t)32 << 20;
hipError_t static_plan_scratch(void** ptr);
size_t attention_state_bytes(int Z, int H, int L);
hipError_t launch_plan(const PlanArgs& a, hipStream_t stream);
hipError_t launch_attention(const AttnArgs& a, hipStream_t stream);
// Debug check of q_perm / kv_perm ranges (allocates, synchronises `stream`); bits: 1 = Q_perm, 2 = KV_perm
hipError_t validate_maps(const AttnArgs& a, hipStream_t stream, int* bits);
// Alg. 2 alone (local.hip): own-segment pass in original query order into the state buffers
hipError_t launch_local(const AttnArgs& a, hipStream_t stream);
// Alg. 3 alone (prefix.hip): prefix walk in permuted query order from the state buffers
hipError_t launch_prefix(const AttnArgs& a, hipStream_t stream);

}  // namespace s2o
