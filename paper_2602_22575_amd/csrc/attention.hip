// S2O sparse attention for gfx950 (paper Sec. 3.2-3.3; Alg. 2 + Alg. 3, Alg. 4 when the
// query order is the identity).
//
// One workgroup = 8 wavefronts = 4 permuted query tiles (4 x 64 rows) of one
// (batch, head, segment); a query tile is owned by a pair of wavefronts, 32 rows each.
// All query tiles of a segment walk the same KV_perm row, so the workgroup stages each
// gathered 64-token K/V tile in LDS once and the eight wavefronts share it.  A wavefront
// keeps its Q fragments, online-softmax state and output accumulator in registers (under
// 256, so two wavefronts fit on a SIMD and one's softmax overlaps the other's MFMAs).  The
// early-stop decision of a query tile is the OR of its two wavefronts' "keep" votes,
// exchanged through LDS at the one workgroup barrier per key tile; the branch is uniform
// per wavefront and is taken one tile late (the PV product of a tile waits for its vote).  The
// dense intra-segment causal window (Pass-1) is run by the same loop before the prefix
// walk, with identity indices and a per-element causal mask, so its state never leaves
// registers.  (That is the single-launch form, used when the caller gives no state buffer;
// with one, the own-segment pass and the prefix walk run as kernels of their own, local.hip
// and prefix.hip.)
//
// MFMA formulation, LDS layouts and the base-2 online softmax with lazy rescaling are in
// attn_tile.h.
#include "attn_tile.h"
#include "s2o_internal.h"

namespace s2o {

namespace {

using namespace tile;

constexpr int kWaves = 8;        // a query tile of B_M rows is B_M/32 wavefronts: 4 tiles of 64
                                 // rows or 2 tiles of 128 rows per workgroup
constexpr int kThreads = 64 * kWaves;
constexpr int kKsElems = kTileElems;
constexpr int kVtElems = kTileElems;
constexpr size_t kAttnLds = (size_t)(2 * kKsElems + 3 * kVtElems) * 2 + 256;

__device__ inline int wave_max_i32(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = max(v, __shfl_xor(v, o));
  return v;
}

// Everything in one launch: own-segment window, then the prefix walk.  (The two-launch form
// costs a round trip of the fp32 state through HBM but halves the own-segment work: a
// permuted query tile needs every own-segment key tile with a per-element mask, a tile in
// original order only those up to its diagonal.)
__global__ __launch_bounds__(kThreads, 1) void s2o_attention_kernel(const AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* Ks = reinterpret_cast<uint16_t*>(smem);
  uint16_t* Vt = Ks + 2 * kKsElems;
  int* sflag = reinterpret_cast<int*>(Vt + 3 * kVtElems);   // [0..7] pmax, [8..23] stop votes (two sets)

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m_ = lane & 31, hh = lane >> 5;
  const int G = a.H / a.Hkv;
  const int BM = a.BM;                                   // query tile rows: 64 or 128
  const int wpt = BM / kRowsPerWave;                     // wavefronts per query tile
  const int tpw = kWaves / wpt;                          // query tiles per workgroup
  const int TJ = a.S / BM;                               // query tiles per segment
  const int JG = (TJ + tpw - 1) / tpw;                   // workgroups per (z,h,n)

  int zh_, nr, jg;
  map_block(blockIdx.x, a.Z * a.H, JG, zh_, nr, jg);
  const int n = a.N - 1 - nr, z = zh_ / a.H, h = zh_ % a.H;
  const int g = h / G;
  const uint16_t* Qh = a.Q + z * a.qs[0] + h * a.qs[1];
  const uint16_t* Kh = a.K + z * a.ks[0] + g * a.ks[1];
  const uint16_t* Vh = a.V + z * a.vs[0] + g * a.vs[1];
  uint16_t* Oh = a.O + z * a.os[0] + h * a.os[1];
  const int64_t zh = (int64_t)z * a.H + h;
  const int32_t* kvrow = a.kv_perm + zh * kv_row_offset(a.N, a.S) + kv_row_offset(n, a.S);
  const int nS = n * a.S;
  const int nK_all = nS / kBN;                 // prefix tiles that exist for this segment
  // prefix tiles this launch may walk: at most the budget
  const int nK = a.max_tiles > 0 ? min(nK_all, a.max_tiles) : nK_all;

  // wavefront -> (query tile of the workgroup, 32-row part); the parts of a tile are
  // wavefronts tile, tile + tpw, ...
  const int tile_l = wave % tpw, part = wave / tpw;
  const int j = jg * tpw + tile_l;              // this wavefront's permuted query tile
  bool active = j < TJ;

  // ---- the query row of this lane and its Q fragments
  int qoff;
  bf16x8 qf[8];
  {
    const int r = min(j, TJ - 1) * BM + kRowsPerWave * part + m_;
    qoff = a.use_q_perm ? a.q_perm[(zh * a.N + n) * a.S + r] : r;
    qoff = min(max(qoff, 0), a.S - 1);
    load_q(Qh + (int64_t)(nS + qoff) * a.qs[2], hh, qf);
  }
  const int wave_pmax = active ? wave_max_i32(qoff) : -1;
  if (lane == 0) sflag[wave] = wave_pmax;
  __syncthreads();
  int wg_pmax = -1;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) wg_pmax = max(wg_pmax, sflag[w]);
  // own-segment key tiles this workgroup needs
  const int nloc = wg_pmax / kBN + 1;
  const int ntiles = nloc + nK;

  // ---- loader: wavefronts 0-3 move K, 4-7 move V, 4 groups of 4 rows each per tile
  const bool loads_v = wave >= 4;
  const uint16_t* src = loads_v ? Vh : Kh;
  const int64_t src_stride = loads_v ? a.vs[2] : a.ks[2];
  // token indices of the tile after the one being fetched are read one step ahead, so that a
  // fetch never waits for its own index loads
  int tokn[4];
  auto load_index = [&](int it) {
    int ld[4] = {0, 0, 0, 0};
    if (nK > 0) {                      // one uniform branch; the loads themselves are unconditional
      const int pt = min(max(it - nloc, 0), nK - 1);
#pragma unroll
      for (int gi = 0; gi < 4; ++gi)
        ld[gi] = kvrow[(int64_t)pt * kBN + 16 * (wave & 3) + 4 * gi + (lane >> 4)];
    }
#pragma unroll
    for (int gi = 0; gi < 4; ++gi)
      tokn[gi] = it < nloc ? nS + it * kBN + 16 * (wave & 3) + 4 * gi + (lane >> 4) : ld[gi];
  };
  const uint32_t stride_bytes = (uint32_t)(src_stride * 2);
  const char* gbase[4];                 // per group: head base + this lane's (swizzled) chunk
#pragma unroll
  for (int gi = 0; gi < 4; ++gi)
    gbase[gi] = reinterpret_cast<const char*>(src) + load_chunk_offset(lane, 16 * (wave & 3) + 4 * gi);
  auto load_tile = [&](int it) {       // K tiles alternate between 2 buffers, V tiles between 3
    uint16_t* dst = loads_v ? Vt + (it % 3) * kVtElems : Ks + (it & 1) * kKsElems;
#pragma unroll
    for (int gi = 0; gi < 4; ++gi) {
      const uint32_t tok = (uint32_t)min(max(tokn[gi], 0), a.L - 1);
      load_rows_to_lds(gbase[gi] + (uint64_t)tok * stride_bytes,   // one 64-bit multiply-add
                       dst + (16 * (wave & 3) + 4 * gi) * kRowElems);
    }
    load_index(it + 1);
  };
  Operands op;
  op.init(lane);

  // ---- online-softmax state and output accumulator O^T[d-block]
  float m_ref = -INFINITY, l_run = 0.f;
  f32x16 o[4];
  zero_acc(o);
  int committed = 0, issued = 0;
  const float c2 = a.scale_log2e;

  // values a tile's score step hands to its PV step
  f32x16 s[2];
  TileStats ts;
  auto qk = [&](int kbuf) { qk_tile(Ks + kbuf * kKsElems, op, qf, s); };
  auto pv = [&](int vbuf, const bf16x8 (&pb)[4]) { pv_tile(Vt + vbuf * kVtElems, op, pb, o); };

  load_index(0);
  load_tile(0);
  __syncthreads();

  // Every wavefront runs the same sequence of barriers, one per key tile.  A wavefront whose
  // query tile has stopped (or that has no query tile) drops into a drain loop that only
  // keeps loading tiles for the others, so the hot loops carry no "am I still active" merges.
  int it = 0;
  // ---- tiles folded in unconditionally: the own-segment tiles (Pass-1: dense, causal mask)
  // and, when no stop rule is asked for (stop_mode 2), the prefix tiles as well
  const int nplain = a.stop_mode == 2 ? ntiles : nloc;
  for (; it < nplain; ++it) {
    if (it + 1 < ntiles) load_tile(it + 1);
    const bool own = it < nloc;
    if (own ? it * kBN <= wave_pmax : active) {   // wave_pmax = -1 for a wavefront without a query tile
      qk(it & 1);
      // own-segment tiles always carry the causal mask: the rows of a permuted query tile are
      // scattered over the segment
      ts = own ? softmax_tile<true>(s, c2, m_ref, l_run, it * kBN, qoff, hh)
               : softmax_tile<false>(s, c2, m_ref, l_run, 0, 0, hh);
      bf16x8 pb[4];
      pack_p(s, pb);
      rescale(o, ts.alpha, ts.grow);
      pv(it % 3, pb);
      l_run = ts.prev + ts.mass;
      m_ref = ts.m_use;
      if (!own) { ++committed; ++issued; }
    }
    __syncthreads();
  }
  // ---- prefix tiles in KV_perm order (Pass-2) with the early-stop rule: the query tile
  // continues iff some row's tile mass reaches tau * (mass so far).  The two wavefronts of a
  // tile vote through LDS; the vote on tile k is written before the barrier that ends step k
  // and read at the start of step k+1, so the PV product of tile k runs one step late (next
  // to the scores of tile k+1) and is simply dropped, or folded in as the last one, when the
  // vote says stop.  The statistics (l, m) are advanced speculatively and rolled back on a
  // drop; the accumulator is only ever touched by a tile that is kept.
  bool pending = false;                 // a scored prefix tile waits for its vote
  bf16x8 pb_pend[4];
  float alpha_pend = 1.f, l_save = 0.f, m_save = 0.f;
  bool grow_pend = false;
  auto vote_flags = [&](int step) { return sflag + 8 + 8 * (step & 1); };
  auto publish = [&](int step) {        // after softmax of tile `step`: vote + speculative stats
    const bool keep = __builtin_amdgcn_ballot_w64(ts.mass >= a.tau * ts.prev) != 0ull;
    if (lane == 0) vote_flags(step)[wave] = keep ? 1 : 0;
    l_save = l_run; m_save = m_ref;
    l_run = ts.prev + ts.mass; m_ref = ts.m_use;
    alpha_pend = ts.alpha; grow_pend = ts.grow;
    pack_p(s, pb_pend);
    pending = true;
    ++issued;
  };
  bool wg_done = false;
  if (active && it < ntiles) {
    // first prefix tile: scores only
    if (it + 1 < ntiles) load_tile(it + 1);
    qk(it & 1);
    ts = softmax_tile<false>(s, c2, m_ref, l_run, 0, 0, hh);
    publish(it);
    __syncthreads();
    ++it;
    for (; it < ntiles; ++it) {
      const int* vf = vote_flags(it - 1);
      int votes = 0;
      for (int p2 = 0; p2 < wpt; ++p2) votes |= vf[tile_l + tpw * p2];
      qk(it & 1);
      if (votes == 0) {
        int any = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) any |= vf[w];
        if (a.stop_mode == 0) {
          l_run = l_save; m_ref = m_save;
        } else {
          rescale(o, alpha_pend, grow_pend);
          pv((it - 1) % 3, pb_pend);
          ++committed;
        }
        pending = false;
        wg_done = any == 0;
        break;
      }
      if (it + 1 < ntiles) load_tile(it + 1);
      rescale(o, alpha_pend, grow_pend);
      pv((it - 1) % 3, pb_pend);
      ++committed;
      ts = softmax_tile<false>(s, c2, m_ref, l_run, 0, 0, hh);
      publish(it);
      __syncthreads();
    }
    if (pending) {                                     // the last prefix tile: its vote is visible now
      const int* vf = vote_flags(ntiles - 1);
      int votes = 0;
      for (int p2 = 0; p2 < wpt; ++p2) votes |= vf[tile_l + tpw * p2];
      const bool stop = votes == 0;
      if (stop && a.stop_mode == 0) {
        l_run = l_save; m_ref = m_save;
      } else {
        rescale(o, alpha_pend, grow_pend);
        pv((ntiles - 1) % 3, pb_pend);
        ++committed;
      }
      wg_done = true;
    }
  }
  // ---- drain: keep the tile pipeline fed until every query tile of the workgroup has stopped
  if (!wg_done) {
    for (; it < ntiles; ++it) {
      if (it > nloc) {
        const int* vf = vote_flags(it - 1);
        int any = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) any |= vf[w];
        if (any == 0) break;
      }
      if (it + 1 < ntiles) load_tile(it + 1);
      if (lane == 0) vote_flags(it)[wave] = 0;
      __syncthreads();
    }
  }

  if (j < TJ) {
    {
      // normalise and scatter to the original row
      store_o(Oh + (int64_t)(nS + qoff) * a.os[2], hh, o, 1.0f / l_run);
      if (lane == 0 && part == 0) {
        const int64_t ci = zh * (a.L / BM) + (int64_t)n * TJ + j;
        if (a.computed) a.computed[ci] = committed;
        if (a.skipped) a.skipped[ci] = nK_all - issued;
      }
    }
  }
}

}  // namespace

size_t attention_state_bytes(int Z, int H, int L) {
  return (size_t)Z * H * L * (kD + 2) * sizeof(float);
}

// ---- debug check of the caller's maps (S2O_VALIDATE_MAPS): bit 0 = a Q_perm entry outside
// [0, S), bit 1 = a KV_perm entry of segment n outside its row's range ([0, n*S); [0, L) without
// causality).  Permutation-ness is not checked.
__global__ __launch_bounds__(256) void validate_maps_kernel(const AttnArgs a, int32_t* flag) {
  const int64_t zh = blockIdx.y;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const int64_t first = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int bad = 0;
  if (a.use_q_perm && a.q_perm) {
    const int32_t* q = a.q_perm + zh * a.L;
    for (int64_t i = first; i < a.L; i += stride) bad |= (q[i] < 0 || q[i] >= a.S) ? 1 : 0;
  }
  if (a.kv_perm) {
    const int64_t total = kv_rows_total(a.N, a.S, a.L, a.non_causal);
    const int32_t* kv = a.kv_perm + zh * total;
    for (int64_t i = first; i < total; i += stride) {
      // segment of packed position i: the largest n with kv_row_start(n) <= i
      int n;
      if (a.non_causal) {
        n = (int)(i / a.L);
      } else {
        n = (int)((1.0 + sqrt(1.0 + 8.0 * (double)(i / a.S))) * 0.5);
        while (kv_row_start(n, a.S, a.L, 0) > i) --n;
        while (kv_row_start(n + 1, a.S, a.L, 0) <= i) ++n;
      }
      const int64_t lim = kv_row_len(n, a.S, a.L, a.non_causal);
      bad |= (kv[i] < 0 || kv[i] >= lim) ? 2 : 0;
    }
  }
  if (bad) atomicOr(flag, bad);
}

hipError_t validate_maps(const AttnArgs& a, hipStream_t stream, int* bits) {
  int32_t* flag = nullptr;
  hipError_t e = hipMalloc(reinterpret_cast<void**>(&flag), sizeof(int32_t));
  if (e != hipSuccess) return e;
  int32_t h = 0;
  e = hipMemcpyAsync(flag, &h, sizeof(h), hipMemcpyHostToDevice, stream);
  if (e == hipSuccess) {
    hipLaunchKernelGGL(validate_maps_kernel, dim3(64, (unsigned)(a.Z * a.H)), dim3(256), 0, stream, a, flag);
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = hipMemcpyAsync(&h, flag, sizeof(h), hipMemcpyDeviceToHost, stream);
  if (e == hipSuccess) e = hipStreamSynchronize(stream);
  (void)hipFree(flag);
  *bits = h;
  return e;
}

hipError_t launch_attention(const AttnArgs& a, hipStream_t stream) {
  if (a.passes != 0) {                 // separate kernels through the state buffers
    if (a.passes & 1) {
      const hipError_t e = launch_local(a, stream);
      if (e != hipSuccess) return e;
    }
    return (a.passes & 2) ? launch_prefix(a, stream) : hipSuccess;
  }
  static std::mutex mu;
  static uint64_t done = 0;
  const hipError_t se = once_per_device(mu, done, [] {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&s2o_attention_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)kAttnLds);
  });
  if (se != hipSuccess) return se;
  const int TJ = a.S / a.BM;
  const int tpw = kWaves / (a.BM / kRowsPerWave);
  const int JG = (TJ + tpw - 1) / tpw;
  const int64_t blocks = (int64_t)a.Z * a.H * a.N * JG;
  if (blocks <= 0 || blocks > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(s2o_attention_kernel, dim3((unsigned)blocks), dim3(kThreads), kAttnLds, stream, a);
  return hipGetLastError();
}

}  // namespace s2o
