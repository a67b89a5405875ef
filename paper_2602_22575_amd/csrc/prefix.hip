// S2O prefix walk (paper Sec. 3.3, Alg. 3; Alg. 4 when the query order is the identity) for
// gfx950, resuming every query row from the state (accumulator, l, m) that the own-segment
// pass (Alg. 2, local.hip) left in the state buffers.
//
// One workgroup = 4 wavefronts = 128 permuted query rows of one (batch, head, segment): two
// query tiles of 64 rows or one of 128, 32 rows per wavefront.  The wavefronts of a segment
// walk the same KV_perm row, so a gathered 64-token K/V tile is staged in LDS once per
// workgroup.  MFMA formulation, LDS layouts, the explicitly scheduled operand reads and the
// base-2 online softmax with lazy rescaling are in attn_tile.h; the early-stop vote is taken
// one tile late, the PV product of a tile waiting for it.
//
// Tile pipeline.  Because the PV product of tile k runs during step k+1, V tile k is only
// needed one step after K tile k, so it is also fetched one step later: step k reads K(k) and
// V(k-1) while K(k+1) and V(k) arrive.  Two K and two V buffers (64 KB) then suffice, and with
// 4 wavefronts of under 256 registers two workgroups share a CU.
// A step is:   read the votes on tile k-1  ->  issue the fetches of K(k+1), V(k) and of the
// token indices of tile k+2  ->  scores of tile k, PV of tile k-1, softmax of tile k  ->  wait
// for the wavefront's own fetches  ->  barrier.  The fetches are issued first and waited for
// last, so they have the whole step to land; nothing between depends on them (the indices
// loaded in step k are first touched at the top of step k+1).
#include "attn_tile.h"
#include "s2o_internal.h"

namespace s2o {

namespace {

using namespace tile;

constexpr int kWaves = 4, kThreads = 64 * kWaves;
constexpr int kKBytes0 = 0, kVBytes0 = 2 * kTileBytes;             // K x2 at 0, V x2 behind them
constexpr size_t kPrefixLds = (size_t)(4 * kTileBytes) + 64 + 4 * kWaves * 64;   // + vote flags + index ring

template <int P> using Par = std::integral_constant<int, P>;

// min(max(x, 0), hi) in one instruction (the compiler emits two: it cannot know that hi >= 0)
__device__ __forceinline__ uint32_t clamp_token(int x, int hi) {
  int r;
  asm("v_med3_i32 %0, %1, 0, %2" : "=v"(r) : "v"(x), "s"(hi));
  return (uint32_t)r;
}

// kNoStop: stop_mode 2 (every prefix tile folded in, the paper's kernel C) as an instantiation
// of its own, so that neither loop's registers weigh on the other.
// kMapped: the walk follows a KV_perm row (always, except the non-causal walk in storage order,
// which then does not carry the map's registers and selects).
template <bool kNoStop, bool kMapped>
__global__ __launch_bounds__(kThreads, 2) void s2o_prefix_kernel(const AttnArgs a) {
  extern __shared__ __attribute__((aligned(256))) unsigned char smem[];   // OperandAddr needs a 256-byte base
  uint16_t* Ks = reinterpret_cast<uint16_t*>(smem);
  uint16_t* Vt = Ks + 2 * kTileElems;
  int* sflag = reinterpret_cast<int*>(Vt + 2 * kTileElems);   // stop votes: two sets of kWaves
  int32_t* ring = reinterpret_cast<int32_t*>(smem + 4 * kTileBytes + 64);   // map entries: 4 tiles x kWaves x 16

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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
  const int32_t* kvrow = a.kv_perm + zh * kv_rows_total(a.N, a.S, a.L, a.non_causal) +
                         kv_row_start(n, a.S, a.L, a.non_causal);
  const int nS = n * a.S;
  // key tiles this segment's row of KV_perm lists: its prefix, or everything without causality
  const int nK_all = (int)(kv_row_len(n, a.S, a.L, a.non_causal) / kBN);
  // prefix tiles this launch may walk: at most the budget
  const int ntiles = a.max_tiles > 0 ? min(nK_all, a.max_tiles) : nK_all;

  // wavefront -> (query tile of the workgroup, 32-row part); the parts of a tile are
  // wavefronts tile, tile + tpw, ...
  const int tile_l = wave % tpw, part = wave / tpw;
  const int j = jg * tpw + tile_l;              // this wavefront's permuted query tile
  const bool active = j < TJ;

  // ---- loader: every wavefront moves 16 rows of K and 16 rows of V per step, 4 rows per
  // instruction (lane l of group gi moves a chunk of tile row 16*wave + 4*gi + l/16).  The map
  // entries of its rows travel through a small ring in LDS, private to the wavefront: the 16
  // entries of tile t+2 are requested (global -> LDS, like the tiles) at the top of step t and
  // first read at the top of step t+1, so no register holds an index across a step and no
  // fetch ever waits for an index load.  Ring position 4*(l/16) + gi holds the entry of row
  // 4*gi + l/16, so a lane gets its four tokens with one 16-byte read.
  const uint32_t k_stride_bytes = (uint32_t)(a.ks[2] * 2), v_stride_bytes = (uint32_t)(a.vs[2] * 2);
  uint32_t goff[4];
#pragma unroll
  for (int gi = 0; gi < 4; ++gi) goff[gi] = (uint32_t)load_chunk_offset(lane, 16 * wave + 4 * gi);
  auto ring_slot = [&](int t) { return ring + (t & 3) * (16 * kWaves) + 16 * wave; };
  // (lane l < 16 requests the entry of tile row 16*wave + 4*(l%4) + l/4)
  auto fetch_index = [&](int t) {       // map entries of tile t (clamped tile number) -> ring; ntiles > 0
    if (kMapped && lane < 16) {
      // scalar base + 32-bit lane offset: no 64-bit per-lane pointer is kept across the walk
      // The lane's offset is worked out again at every call (opaque lane id): kept across the
      // walk it would be a 64-bit per-lane pointer, two registers that the allocator spills
      // and reloads inside the step, behind a wait for every fetch in flight.
      int l = lane;
      asm volatile("" : "+v"(l));
      const uint32_t row4 = (uint32_t)(4 * (16 * wave + 4 * (l & 3) + ((l >> 2) & 3)));
      const char* tile_idx = reinterpret_cast<const char*>(kvrow + (int64_t)min(t, ntiles - 1) * kBN);
      __builtin_amdgcn_global_load_lds((const gvoid*)(tile_idx + (uint64_t)row4), (lvoid*)ring_slot(t), 4, 0, 0);
    }
  };
  auto tokens = [&](int t, uint32_t (&tok)[4]) {   // this lane's four tokens of tile t, clamped to the sequence
    if (kMapped) {
      const int4 e = *reinterpret_cast<const int4*>(ring_slot(t) + 4 * (lane >> 4));
      const int ev[4] = {e.x, e.y, e.z, e.w};
#pragma unroll
      for (int gi = 0; gi < 4; ++gi) tok[gi] = clamp_token(ev[gi], a.L - 1);
    } else {                            // no map (non-causal only): the keys in storage order
#pragma unroll
      for (int gi = 0; gi < 4; ++gi)
        tok[gi] = (uint32_t)min(min(t, ntiles - 1) * kBN + 16 * wave + 4 * gi + (lane >> 4), a.L - 1);
    }
  };
  auto load_k = [&](int t, const uint32_t (&tok)[4]) {   // K tile t -> buffer t & 1
    uint16_t* kd = Ks + (t & 1) * kTileElems;
#pragma unroll
    for (int gi = 0; gi < 4; ++gi)
      load_rows_to_lds(reinterpret_cast<const char*>(Kh) + (uint64_t)(__umul24(tok[gi], k_stride_bytes) + goff[gi]),
                       kd + (16 * wave + 4 * gi) * kRowElems);
  };
  auto load_v = [&](int t, const uint32_t (&tok)[4]) {   // V tile t -> buffer t & 1
    uint16_t* vd = Vt + (t & 1) * kTileElems;
#pragma unroll
    for (int gi = 0; gi < 4; ++gi)
      load_rows_to_lds(reinterpret_cast<const char*>(Vh) + (uint64_t)(__umul24(tok[gi], v_stride_bytes) + goff[gi]),
                       vd + (16 * wave + 4 * gi) * kRowElems);
  };
  // the fetches of step t (top of the step): K(t+1), V(t) (no stop rule: V(t+1)), indices of tile t+2
  // A wavefront calls fetch_step for t = 0, 1, 2, ... in turn (working or draining), so the
  // tokens of tile t, which V(t) needs, are the ones the previous call worked out for K(t):
  // they stay in four registers instead of being read from the ring and clamped again.
  uint32_t tok_cur[4] = {0, 0, 0, 0};
  auto fetch_step = [&](int t) {
    uint32_t tn[4];
    tokens(t + 1, tn);
    if (kNoStop) {
      if (t + 1 < ntiles) { load_k(t + 1, tn); load_v(t + 1, tn); }
    } else {
      if (t + 1 < ntiles) load_k(t + 1, tn);
      load_v(t, tok_cur);
#pragma unroll
      for (int gi = 0; gi < 4; ++gi) tok_cur[gi] = tn[gi];
    }
    fetch_index(t + 2);
  };
  if (ntiles > 0) {
    fetch_index(0);
    fetch_index(1);
    wait_tile_loads();
    tokens(0, tok_cur);
    load_k(0, tok_cur);
    if (kNoStop) load_v(0, tok_cur);
  }

  // ---- the query row of this lane and its Q fragments
  int qoff;
  bf16x8 qf[8];
  {
    const int r = min(j, TJ - 1) * BM + kRowsPerWave * part + m_;
    qoff = a.use_q_perm ? a.q_perm[(zh * a.N + n) * a.S + r] : r;
    qoff = min(max(qoff, 0), a.S - 1);
    load_q(Qh + (int64_t)(nS + qoff) * a.qs[2], hh, qf);
  }
  OperandAddr oa;
  oa.init(lane, lds_address(smem));

  // ---- online-softmax state and output accumulator O^T[d-block], resumed from the state
  // buffers (row (z, h, l) -> accumulator, l, m).  The statistics are needed by the first
  // softmax; the accumulator only by the first PV product, one step later: its 512 bytes per
  // row are requested after the first tile's scores have been issued and arrive behind them.
  const float c2 = a.scale_log2e;
  // Without causality there is no own-segment pass: every row starts from the empty state.
  const int64_t st_row = zh * a.L + nS + qoff;
  float m_ref = -INFINITY, l_run = 0.f;
  if (!a.non_causal) { m_ref = a.st_m[st_row]; l_run = a.st_l[st_row]; }
  f32x16 o[4];
  const float* st_acc_row = a.st_acc + st_row * kD + 16 * hh;
  auto init_acc = [&] {
    if (a.non_causal) zero_acc(o);
    else load_acc(st_acc_row, o);
  };
  int committed = 0, issued = 0;

  f32x16 s[2];
  TileStats ts;
  auto softmax = [&] { ts = softmax_tile<false>(s, c2, m_ref, l_run, 0, 0, hh); };

  // ---- prefix tiles in KV_perm order with the early-stop rule: the query tile continues iff
  // some row's tile mass reaches tau * (mass so far).  The wavefronts of a tile vote through
  // LDS; the vote on tile k is written before the barrier that ends step k and read at the
  // start of step k+1, where the PV product of tile k is then run, dropped, or folded in as
  // the last one.  The statistics (l, m) are advanced speculatively and rolled back on a
  // drop; the accumulator is only ever touched by a tile that is kept.  Every wavefront runs
  // one barrier per step; one whose query tile has stopped (or that has none) drops into a
  // drain loop that only keeps fetching tiles for the others.
  bf16x8 pb_pend[4];
  float alpha_pend = 1.f, l_save = 0.f, m_save = 0.f;
  bool grow_pend = false;
  auto vote_flags = [&](int step) { return sflag + kWaves * (step & 1); };
  auto publish = [&](int step) {        // after softmax of tile `step`: vote + speculative stats
    const bool keep = __builtin_amdgcn_ballot_w64(ts.mass >= a.tau * ts.prev) != 0ull;
    if (lane == 0) vote_flags(step)[wave] = keep ? 1 : 0;
    l_save = l_run; m_save = m_ref;
    l_run = ts.prev + ts.mass; m_ref = ts.m_use;
    alpha_pend = ts.alpha; grow_pend = ts.grow;
    pack_p(s, pb_pend);
    ++issued;
  };
  // the four wavefronts' votes of a step come with one 16-byte read; a query tile's wavefronts
  // are tile_l, tile_l + tpw, ...
  struct Votes { int mine, any; };
  // (The read sits in a loop of one trip whose count the compiler cannot see.  Without an inner
  // loop in the step, the step loop is the innermost one, the compiler hoists and schedules far
  // more aggressively, and the walk ends up with 256 registers and spill reloads -- each behind
  // a wait for all fetches in flight -- inside the step: 158 against 110 ms for the dense walk.)
  const int one_trip = 1 + (a.BM >> 12);
  auto read_votes = [&](int step) {
    Votes v = {0, 0};
    for (int trip = 0; trip < one_trip; ++trip) {
      const int4 f = *reinterpret_cast<const int4*>(vote_flags(step) + 4 * trip);
      v.any |= __builtin_amdgcn_readfirstlane(f.x | f.y | f.z | f.w);
      v.mine |= tpw == 2 ? __builtin_amdgcn_readfirstlane(tile_l == 0 ? (f.x | f.z) : (f.y | f.w)) : v.any;
    }
    return v;
  };
  auto end_step = [&] {                 // this wavefront's fetches have landed; everyone's after the barrier
    wait_tile_loads();
    __syncthreads();
  };

  bool acc_loaded = false;
  if (kNoStop && ntiles > 0) {
    // ---- every prefix tile is folded in (no votes, nothing deferred): step k reads K(k) and
    // V(k) while K(k+1) and V(k+1) arrive
    end_step();                                   // K and V tile 0 have landed
    auto plain_step = [&](auto par_, int it) {
      constexpr int P = decltype(par_)::value;
      fetch_step(it);
      if (active) {
        qk_tile_only<kKBytes0 + P * kTileBytes>(oa, qf, s);
        if (!acc_loaded) { init_acc(); acc_loaded = true; }
        softmax();
        pack_p(s, pb_pend);
        rescale(o, ts.alpha, ts.grow);
        pv_tile_only<kVBytes0 + P * kTileBytes>(oa, pb_pend, o);
        l_run = ts.prev + ts.mass; m_ref = ts.m_use;
        ++committed; ++issued;
      }
      end_step();
    };
    for (int it = 0; it < ntiles; it += 2) {
      plain_step(Par<0>{}, it);
      if (it + 1 < ntiles) plain_step(Par<1>{}, it + 1);
    }
  } else if (ntiles > 0) {
    end_step();                                   // K tile 0 has landed
    int it = 0;
    bool wg_done = false;
    if (active) {
      // first tile: scores only
      fetch_step(0);
      qk_tile_only<kKBytes0>(oa, qf, s);
      init_acc(); acc_loaded = true;
      softmax();
      publish(0);
      end_step();
      bool pending = true;                      // a scored tile waits for its vote
      // One step.  K(it) sits in K buffer it & 1, V(it-1) in V buffer (it-1) & 1: the operand
      // addresses `fa` carry the current buffers and are moved to the other buffers at the end of
      // every completed step (sixteen additions, outside the sequence of reads and MFMAs), so one
      // loop body serves both parities -- two bodies with the buffer as a constant get the
      // accumulator different registers and pay a 32-move shuffle between them on every step.
      // Returns false when the query tile stops at this step.
      OperandAddr fa = oa.at((uint32_t)(kKBytes0 + kTileBytes), (uint32_t)kVBytes0);   // step 1
      auto step = [&](int it_) -> bool {
        const Votes vf = read_votes(it_ - 1);
        const int votes = vf.mine;
        if (votes == 0) {
          const int any = vf.any;
          if (a.stop_mode == 0) {
            l_run = l_save; m_ref = m_save;
          } else {
            rescale(o, alpha_pend, grow_pend);
            pv_tile_only<0>(fa, pb_pend, o);
            ++committed;
          }
          pending = false;
          wg_done = any == 0;
          return false;
        }
        fetch_step(it_);
        u32x2 vfr[16][2];
        qk_tile_sched<0, 0, true>(fa, qf, s, vfr);
        rescale(o, alpha_pend, grow_pend);
        pv_tile_sched<0, true>(fa, pb_pend, o, vfr);
        ++committed;
        bool redo;
        ts = softmax_tile_keep_reference(s, c2, m_ref, l_run, redo);
        if (__builtin_amdgcn_ballot_w64(redo) != 0ull) {   // rare: the tile moves some row's reference
          qk_tile_only<0>(fa, qf, s);
          softmax();
        }
        publish(it_);
        {                                       // step it_ + 1: K moves to the other buffer, V the other way
          const uint32_t dk = (it_ & 1) ? (uint32_t)(-kTileBytes) : (uint32_t)kTileBytes;
          fa.shift(dk, 0u - dk);
        }
        wait_tile_loads();
        __syncthreads();
        return true;
      };
      for (it = 1; it < ntiles; ++it)
        if (!step(it)) break;
      if (pending) {                            // the last tile: its vote is visible now
        const bool stop = read_votes(ntiles - 1).mine == 0;
        if (stop && a.stop_mode == 0) {
          l_run = l_save; m_ref = m_save;
        } else {
          rescale(o, alpha_pend, grow_pend);
          pv_tile_only<0>(fa, pb_pend, o);      // fa stands at step ntiles: V(ntiles-1)
          ++committed;
        }
        wg_done = true;
      }
    }
    // ---- drain: keep the tile pipeline fed until every query tile of the workgroup has stopped
    if (!wg_done) {
      for (; it < ntiles; ++it) {
        if (it > 0 && read_votes(it - 1).any == 0) break;
        fetch_step(it);
        if (lane == 0) vote_flags(it)[wave] = 0;
        end_step();
      }
    }
  }

  if (active) {
    if (!acc_loaded) init_acc();                 // no prefix tile was walked (first segment)
    // normalise and scatter to the original row
    // (every wavefront of the workgroup is past the last barrier: the K buffers are idle)
    store_o_rows(Oh, a.os[2], nS + qoff, smem + wave * 8192, lane, o, 1.0f / l_run);
    if (lane == 0 && part == 0) {
      const int64_t ci = zh * (a.L / BM) + (int64_t)n * TJ + j;
      if (a.computed) a.computed[ci] = committed;
      if (a.skipped) a.skipped[ci] = nK_all - issued;
    }
  }
}

}  // namespace

hipError_t launch_prefix(const AttnArgs& a, hipStream_t stream) {
  static std::mutex mu;
  static uint64_t done = 0;
  const hipError_t se = once_per_device(mu, done, [] {
    const void* fns[4] = {reinterpret_cast<const void*>(&s2o_prefix_kernel<false, true>),
                          reinterpret_cast<const void*>(&s2o_prefix_kernel<true, true>),
                          reinterpret_cast<const void*>(&s2o_prefix_kernel<false, false>),
                          reinterpret_cast<const void*>(&s2o_prefix_kernel<true, false>)};
    for (const void* f : fns) {
      const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kPrefixLds);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  });
  if (se != hipSuccess) return se;
  const int TJ = a.S / a.BM;
  const int tpw = kWaves / (a.BM / kRowsPerWave);
  const int JG = (TJ + tpw - 1) / tpw;
  const int64_t blocks = (int64_t)a.Z * a.H * a.N * JG;
  if (blocks <= 0 || blocks > 0x7fffffff) return hipErrorInvalidValue;
  const dim3 grid((unsigned)blocks), block(kThreads);
  if (a.kv_perm) {
    if (a.stop_mode == 2) hipLaunchKernelGGL((s2o_prefix_kernel<true, true>), grid, block, kPrefixLds, stream, a);
    else hipLaunchKernelGGL((s2o_prefix_kernel<false, true>), grid, block, kPrefixLds, stream, a);
  } else {
    if (a.stop_mode == 2) hipLaunchKernelGGL((s2o_prefix_kernel<true, false>), grid, block, kPrefixLds, stream, a);
    else hipLaunchKernelGGL((s2o_prefix_kernel<false, false>), grid, block, kPrefixLds, stream, a);
  }
  return hipGetLastError();
}

}  // namespace s2o
