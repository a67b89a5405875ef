// S2O own-segment pass (paper Sec. 3.2, Alg. 2) for gfx950: dense causal attention of every
// query over the keys of its own segment, queries in original order, leaving the
// un-normalised online-softmax state (accumulator, l, m) per row for the prefix walk.
//
// A row block = 128 consecutive query rows of one (batch, head, segment), 32 rows per
// wavefront; it needs the key tiles 0 .. (its last row) / 64 of the segment and the causal
// mask only where a row ends inside a tile.  One workgroup = 4 wavefronts takes two row
// blocks in turn, one of the upper and one of the lower half of the segment; the second
// block's first tile and query rows are fetched under the first block's last tile.  Nothing
// here depends on the query tile size or on the index maps.  With K and V double-buffered a
// workgroup takes 64 KB of LDS and 4 wavefronts of at most 256 registers, so two workgroups
// share a CU: their barriers are independent, and one's prologue and epilogue overlap the
// other's tiles.
//
// The state (2 KB per row) is written as whole 128-byte lines, regrouped through the tile
// buffers that are idle at the end of a block (attn_tile.h, lines_from_acc), and the next
// block's first fetches are issued in front of those stores: memory instructions complete in
// order, so the next barrier can wait for the fetches and leave the stores in flight.
//
// MFMA formulation, LDS layouts and the base-2 online softmax with lazy rescaling are in
// attn_tile.h.
#include "attn_tile.h"
#include "s2o_internal.h"

namespace s2o {

namespace {

using namespace tile;

constexpr int kWaves = 4, kThreads = 64 * kWaves;
constexpr int kRowsPerWg = kWaves * kRowsPerWave;
constexpr size_t kLocalLds = (size_t)(4 * kTileElems) * 2;   // K x2, V x2
constexpr int kStateStores = 16;   // store instructions a wavefront needs at least for its 16 KB of state

// The end-of-step wait and barrier.  Tiles reach LDS by global->LDS loads only, so the barrier
// needs the vector-memory counter and no LDS fence; the fragment reads of a step are all
// consumed by its MFMAs before the wavefront gets here.  The wait goes through the builtin so
// that the compiler's own bookkeeping of outstanding loads sees it.
template <int kYoungest>
__device__ __forceinline__ void wait_fetches() {
  // s_waitcnt immediate: vmcnt in bits 3..0 and 15..14, every other counter left at its maximum
  __builtin_amdgcn_s_waitcnt((kYoungest & 15) | ((kYoungest >> 4) << 14) | 0x0f70);
  asm volatile("" ::: "memory");
}
__device__ __forceinline__ void tile_barrier() { asm volatile("s_barrier" ::: "memory"); }

__global__ __launch_bounds__(kThreads, 2) void s2o_local_kernel(const AttnArgs a) {
  extern __shared__ __attribute__((aligned(256))) unsigned char smem[];   // OperandAddr needs a 256-byte base
  uint16_t* Ks = reinterpret_cast<uint16_t*>(smem);
  uint16_t* Vt = Ks + 2 * kTileElems;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: branches on it are scalar
  const int m_ = lane & 31, hh = lane >> 5;
  const int G = a.H / a.Hkv;
  const int JG = (a.S + kRowsPerWg - 1) / kRowsPerWg;   // row blocks of 128 per (z,h,n)
  const int PG = (JG + 1) / 2;                          // workgroups per (z,h,n): a long and a short block each

  // Workgroup -> (z, KV head, segment, query head of the group, pos).  Every (z, KV head, segment)
  // is one unit of G * PG workgroups with consecutive ids on one XCD (block ids are dealt
  // round-robin to the 8 XCDs), the G query heads of the group interleaved: they read the same
  // 2 * S rows of K and V at about the same time, so the segment is fetched from HBM once per
  // group instead of once per query head.  All units cost the same here (no early stop), so
  // nothing needs balancing across XCDs.
  int z, g, n, h, pos;
  {
    const int per_unit = G * PG, U = a.Z * a.Hkv * a.N, b = blockIdx.x;
    int u, within;
    if (U % 8 == 0) {
      const int xcd = b & 7, idx = b >> 3;
      u = (idx / per_unit) * 8 + xcd;
      within = idx % per_unit;
    } else {
      u = b / per_unit;
      within = b % per_unit;
    }
    pos = within / G;
    n = u % a.N;
    g = (u / a.N) % a.Hkv;
    z = u / (a.N * a.Hkv);
    h = g * G + within % G;
  }
  const uint16_t* Qh = a.Q + z * a.qs[0] + h * a.qs[1];
  const uint16_t* Kh = a.K + z * a.ks[0] + g * a.ks[1];
  const uint16_t* Vh = a.V + z * a.vs[0] + g * a.vs[1];
  const int64_t zh = (int64_t)z * a.H + h;
  const int nS = n * a.S;
  // row blocks JG-1-pos and JG/2-1-pos, the longest pair first: workgroups of different length
  // drift apart, so that the two on a CU are rarely both at a block's end (state stores, no
  // MFMA work) at once; the middle block of an odd JG stands alone
  const int jg_of[2] = {JG - 1 - pos, JG / 2 - 1 - pos};
  const int nblk = jg_of[1] < 0 ? 1 : 2;

  // ---- loader: every wavefront moves 16 rows of K and 16 rows of V per tile, 4 rows per
  // instruction (scalar base + 32-bit lane offset: a head spans less than 4 GiB).  The tiles of
  // the workgroup's whole run (both row blocks) are numbered g = 0, 1, ...; K(g) and V(g) sit in
  // buffer g & 1 of their kind.
  const uint32_t k_stride_bytes = (uint32_t)(a.ks[2] * 2), v_stride_bytes = (uint32_t)(a.vs[2] * 2);
  int goff[4];
#pragma unroll
  for (int gi = 0; gi < 4; ++gi) goff[gi] = load_chunk_offset(lane, 16 * wave + 4 * gi);
  auto load_k = [&](int tile, int buf) {
    uint16_t* kd = Ks + buf * kTileElems;
#pragma unroll
    for (int gi = 0; gi < 4; ++gi) {
      const uint32_t tok = (uint32_t)min(nS + tile * kBN + 16 * wave + 4 * gi + (lane >> 4), a.L - 1);
      uint32_t off = __umul24(tok, k_stride_bytes) + goff[gi];
      asm volatile("" : "+v"(off));         // stays a 32-bit offset from the scalar base
      load_rows_to_lds(reinterpret_cast<const char*>(Kh) + (uint64_t)off,
                       kd + (16 * wave + 4 * gi) * kRowElems);
    }
  };
  auto load_v = [&](int tile, int buf) {
    uint16_t* vd = Vt + buf * kTileElems;
#pragma unroll
    for (int gi = 0; gi < 4; ++gi) {
      const uint32_t tok = (uint32_t)min(nS + tile * kBN + 16 * wave + 4 * gi + (lane >> 4), a.L - 1);
      uint32_t off = __umul24(tok, v_stride_bytes) + goff[gi];
      asm volatile("" : "+v"(off));         // stays a 32-bit offset from the scalar base
      load_rows_to_lds(reinterpret_cast<const char*>(Vh) + (uint64_t)off,
                       vd + (16 * wave + 4 * gi) * kRowElems);
    }
  };
  load_k(0, 0);

  // rows of this wavefront in block jg: r0 .. r0 + 31 (original order), all inside the
  // segment or none (S is a multiple of 64, r0 of 32)
  auto row0 = [&](int jg) { return jg * kRowsPerWg + kRowsPerWave * wave; };
  auto row_of = [&](int jg) { return min(row0(jg) + m_, a.S - 1); };
  auto tiles_of = [&](int jg) { return (min(jg * kRowsPerWg + kRowsPerWg, a.S) - 1) / kBN + 1; };
  bf16x8 qf[8];
  load_q(Qh + (int64_t)(nS + row_of(jg_of[0])) * a.qs[2], hh, qf);
  OperandAddr oa;
  oa.init(lane, lds_address(smem));
  // operand addresses for step g: K(g) in K buffer g & 1, V(g-1) in V buffer (g-1) & 1 (K x2 at
  // LDS offset 0, V x2 behind them)
  auto aim = [&](int g_) {
    return oa.at((uint32_t)((g_ & 1) * kTileBytes), (uint32_t)((2 + ((g_ - 1) & 1)) * kTileBytes));
  };

  const float c2 = a.scale_log2e;
  f32x16 o[4];
  f32x16 s[2];
  int gstep = 0;                                // tiles the workgroup has walked so far
  // The accumulator state of a block leaves during step 0 of the next block (`carry`: o then
  // holds it regrouped into lines; the PV products of the new block only start with step 1).
  bool carry = false;
  float* carry_rows = nullptr;

  wait_fetches<0>();
  tile_barrier();                               // K tile 0 has landed

  // The PV product of a tile runs one step late, next to the scores of the following tile (as
  // in the prefix walk): the MFMAs of PV(t-1) do not depend on the softmax of tile t, so its
  // exponentials run in their shadow instead of between two MFMA bursts.  V is therefore also
  // fetched one step late: step g reads K(g) and V(g-1) while K(g+1) and V(g) arrive.
  for (int bi = 0; bi < nblk; ++bi) {
    const int jg = jg_of[bi];
    const int r0 = row0(jg);
    const bool active = r0 < a.S;
    const int qoff = row_of(jg);
    const int wave_pmax = active ? min(r0 + kRowsPerWave - 1, a.S - 1) : -1;
    const int nloc = tiles_of(jg);              // key tiles this block needs
    const int myn = active ? wave_pmax / kBN + 1 : 0;   // ... and this wavefront
    const bool more = bi + 1 < nblk;
    float m_ref = -INFINITY, l_run = 0.f;
    if (!carry) zero_acc(o);
    bf16x8 pb_pend[4];
    float alpha_pend = 1.f;
    bool grow_pend = false, pending = false;

    // softmax of the scores in s -> the tile waiting for its PV product
    auto softmax_step = [&](int it) {
      // CausalMask only if some row of the wavefront ends inside this tile
      const bool masked = it * kBN + kBN - 1 > r0;
      const TileStats t = masked ? softmax_tile<true>(s, c2, m_ref, l_run, it * kBN, qoff, hh)
                                 : softmax_tile<false>(s, c2, m_ref, l_run, it * kBN, qoff, hh);
      pack_p(s, pb_pend);
      alpha_pend = t.alpha; grow_pend = t.grow;
      l_run = t.prev + t.mass;
      m_ref = t.m_use;
      pending = true;
    };
    // K of the block's next tile, else tile 0: of the next block (same segment), or unused.
    // Always eight fetch instructions: the compiler's wait for the Q rows, loaded between two
    // blocks, then never reaches into a step's own fetches.
    auto fetch_step = [&](int it) {
      load_k(it + 1 < nloc ? it + 1 : 0, (gstep + 1) & 1);
      load_v(it, gstep & 1);
    };

    int it = 0;
    if (carry) {
      // Step 0 behind another block: no PV product yet, so o still holds that block's state.  It
      // leaves behind this step's fetches.  Memory instructions complete in order: the wait for
      // all but the kStateStores youngest covers the fetches and leaves the stores in flight.
      wait_fetches<0>();                        // the Q rows, requested before the last PV product
      fetch_step(0);
      if (myn > 0) {
        qk_tile_only<0>(aim(gstep), qf, s);
        softmax_step(0);
      }
      store_acc_lines(carry_rows, o, lane);
      zero_acc(o);
      carry = false;
      wait_fetches<kStateStores>();
      tile_barrier();
      it = 1; ++gstep;
    } else {
      wait_fetches<0>();                        // (a wait on every path into the loop: see wait_fetches)
    }
    for (; it < nloc; ++it, ++gstep) {
      fetch_step(it);
      const OperandAddr fa = aim(gstep);
      if (it < myn) {
        if (pending) {
          u32x2 vfr[16][2];
          qk_tile_sched<0, 0, true>(fa, qf, s, vfr);
          rescale(o, alpha_pend, grow_pend);
          pv_tile_sched<0, true>(fa, pb_pend, o, vfr);
        } else {
          qk_tile_only<0>(fa, qf, s);
        }
        softmax_step(it);
      } else if (pending) {                     // this wavefront's last tile, one step after its scores
        rescale(o, alpha_pend, grow_pend);
        pv_tile_only<0>(fa, pb_pend, o);
        pending = false;
      }
      wait_fetches<0>();                        // this wavefront's part of the fetches has landed
      tile_barrier();
    }

    // ---- leave the un-normalised state for the prefix walk
    if (active && hh == 0) {
      const int64_t st_row = zh * a.L + nS + qoff;
      a.st_l[st_row] = l_run;
      a.st_m[st_row] = m_ref;
    }
    // the next block's query rows, under the last PV product and the state's way out
    if (more) load_q(Qh + (int64_t)(nS + row_of(jg_of[bi + 1])) * a.qs[2], hh, qf);
    if (pending) {                              // the block's last tile: its V arrived during the last step
      const OperandAddr fa = aim(gstep);
      rescale(o, alpha_pend, grow_pend);
      pv_tile_only<0>(fa, pb_pend, o);
    }
    // K buffer (gstep-1) & 1 and V buffer gstep & 1 were last read before the block's last
    // barrier: a quarter of each per wavefront regroups the accumulators into whole lines.  Both
    // are the targets of the next step's fetches, which therefore wait for every wavefront to be
    // through with them.
    float* rows = a.st_acc + (zh * a.L + nS + r0) * kD;
    if (active)
      lines_from_acc(o, lds_address(smem) + ((gstep - 1) & 1) * kTileBytes + wave * 4096,
                     lds_address(smem) + (2 + (gstep & 1)) * kTileBytes + wave * 4096, lane);
    if (more) {
      asm volatile("s_barrier" ::: "memory");   // (lines_from_acc has waited for its LDS reads)
      carry = active;
      carry_rows = rows;
    } else if (active) {
      store_acc_lines(rows, o, lane);
    }
  }
}

}  // namespace

hipError_t launch_local(const AttnArgs& a, hipStream_t stream) {
  static std::mutex mu;
  static uint64_t done = 0;
  const hipError_t se = once_per_device(mu, done, [] {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&s2o_local_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLocalLds);
  });
  if (se != hipSuccess) return se;
  const int JG = (a.S + kRowsPerWg - 1) / kRowsPerWg;
  const int64_t blocks = (int64_t)a.Z * a.H * a.N * ((JG + 1) / 2);
  if (blocks <= 0 || blocks > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(s2o_local_kernel, dim3((unsigned)blocks), dim3(kThreads), kLocalLds, stream, a);
  return hipGetLastError();
}

}  // namespace s2o
