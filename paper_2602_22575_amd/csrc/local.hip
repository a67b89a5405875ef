// S2O own-segment pass (paper Sec. 3.2, Alg. 2) for gfx950: dense causal attention of every
// query over the keys of its own segment, queries in original order, leaving the
// un-normalised online-softmax state (accumulator, l, m) per row for the prefix walk.
//
// A row block = 128 consecutive query rows of one (batch, head, segment), 32 rows per
// wavefront; it needs the key tiles 0 .. (its last row) / 64 of the segment and the causal
// mask only where a row ends inside a tile.  One workgroup = 4 wavefronts takes two row
// blocks in turn, a long one and a short one (blocks JG-1-p and p of the segment), so that
// every workgroup walks the same number of key tiles and the second block's first tile and
// query rows are fetched under the first block's last tile, its state stores issued under
// the second block's scores (own-segment pass 3.30 -> 3.16 ms at 128K against one block per
// workgroup).  Nothing here depends on the query tile size or on the index maps.  With K and
// V double-buffered a workgroup takes 64 KB of LDS and 4 wavefronts of at most 256
// registers, so two workgroups share a CU: their barriers are independent, and one's
// prologue and epilogue (2 KB of state per row) overlap the other's tiles.
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

__global__ __launch_bounds__(kThreads, 2) void s2o_local_kernel(const AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* Ks = reinterpret_cast<uint16_t*>(smem);
  uint16_t* Vt = Ks + 2 * kTileElems;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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
  // row blocks JG-1-pos and pos: together 2*JG + 2 key tiles whatever pos is, so all
  // workgroups of a launch run equally long; the middle block of an odd JG stands alone
  const int jg_of[2] = {JG - 1 - pos, pos};
  const int nblk = jg_of[0] == jg_of[1] ? 1 : 2;

  // ---- loader: every wavefront moves 16 rows of K and 16 rows of V per tile, 4 rows per
  // instruction; `slot` alternates over the whole run of the workgroup
  const uint32_t k_stride_bytes = (uint32_t)(a.ks[2] * 2), v_stride_bytes = (uint32_t)(a.vs[2] * 2);
  int goff[4];
#pragma unroll
  for (int gi = 0; gi < 4; ++gi) goff[gi] = load_chunk_offset(lane, 16 * wave + 4 * gi);
  auto load_tile = [&](int tile, int slot) {
    uint16_t* kd = Ks + slot * kTileElems;
    uint16_t* vd = Vt + slot * kTileElems;
#pragma unroll
    for (int gi = 0; gi < 4; ++gi) {
      const uint32_t tok = (uint32_t)min(nS + tile * kBN + 16 * wave + 4 * gi + (lane >> 4), a.L - 1);
      load_rows_to_lds(reinterpret_cast<const char*>(Kh) + (uint64_t)tok * k_stride_bytes + goff[gi],
                       kd + (16 * wave + 4 * gi) * kRowElems);
      load_rows_to_lds(reinterpret_cast<const char*>(Vh) + (uint64_t)tok * v_stride_bytes + goff[gi],
                       vd + (16 * wave + 4 * gi) * kRowElems);
    }
  };
  load_tile(0, 0);

  // rows of this wavefront in block jg: r0 .. r0 + 31 (original order), all inside the
  // segment or none (S is a multiple of 64, r0 of 32)
  auto row0 = [&](int jg) { return jg * kRowsPerWg + kRowsPerWave * wave; };
  auto row_of = [&](int jg) { return min(row0(jg) + m_, a.S - 1); };
  bf16x8 qf[8];
  load_q(Qh + (int64_t)(nS + row_of(jg_of[0])) * a.qs[2], hh, qf);
  Operands op;
  op.init(lane);

  const float c2 = a.scale_log2e;
  f32x16 o[4];
  f32x16 s[2];
  int slot = 0;

  __syncthreads();                              // tile 0 has landed

  for (int bi = 0; bi < nblk; ++bi) {
    const int jg = jg_of[bi];
    const int r0 = row0(jg);
    const bool active = r0 < a.S;
    const int qoff = row_of(jg);
    const int wave_pmax = active ? min(r0 + kRowsPerWave - 1, a.S - 1) : -1;
    const int wg_pmax = min(jg * kRowsPerWg + kRowsPerWg, a.S) - 1;
    const int nloc = wg_pmax / kBN + 1;         // key tiles this block needs
    const int myn = active ? wave_pmax / kBN + 1 : 0;   // ... and this wavefront
    const bool more = bi + 1 < nblk;
    float m_ref = -INFINITY, l_run = 0.f;
    zero_acc(o);
    if (more && myn == 0) load_q(Qh + (int64_t)(nS + row_of(jg_of[bi + 1])) * a.qs[2], hh, qf);

    for (int it = 0; it < nloc; ++it, slot ^= 1) {
      // the next tile of this block, or the first tile of the next block
      if (it + 1 < nloc) load_tile(it + 1, slot ^ 1);
      else if (more) load_tile(0, slot ^ 1);
      if (it < myn) {
        qk_tile(Ks + slot * kTileElems, op, qf, s);
        // the Q registers are free after a block's last scores: fetch the next block's rows
        if (more && it == myn - 1) load_q(Qh + (int64_t)(nS + row_of(jg_of[bi + 1])) * a.qs[2], hh, qf);
        // CausalMask only if some row of the wavefront ends inside this tile
        const bool masked = it * kBN + kBN - 1 > r0;
        const TileStats t = masked ? softmax_tile<true>(s, c2, m_ref, l_run, it * kBN, qoff, hh)
                                   : softmax_tile<false>(s, c2, m_ref, l_run, it * kBN, qoff, hh);
        bf16x8 pb[4];
        pack_p(s, pb);
        rescale(o, t.alpha, t.grow);
        pv_tile(Vt + slot * kTileElems, op, pb, o);
        l_run = t.prev + t.mass;
        m_ref = t.m_use;
      }
      __syncthreads();
    }

    if (active) {
      // leave the un-normalised state for the prefix walk
      const int64_t st_row = zh * a.L + nS + qoff;
      store_acc(a.st_acc + st_row * kD + 64 * hh, o);
      if (hh == 0) { a.st_l[st_row] = l_run; a.st_m[st_row] = m_ref; }
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
