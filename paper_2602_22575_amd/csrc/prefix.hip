// S2O prefix walk (paper Sec. 3.3, Alg. 3; Alg. 4 when the query order is the identity) for
// gfx950, resuming every query row from the state (accumulator, l, m) that the own-segment
// pass (Alg. 2, local.hip) left in the state buffers.
//
// One workgroup = 4 wavefronts = 128 permuted query rows of one (batch, head, segment): two
// query tiles of 64 rows or one of 128, 32 rows per wavefront.  The wavefronts of a segment
// walk the same KV_perm row, so a gathered 64-token K/V tile is staged in LDS once per
// workgroup.  MFMA formulation, LDS layouts, the base-2 online softmax with lazy rescaling
// and the early-stop vote (taken one tile late, the PV product of a tile waiting for it) are
// those of attention.hip; see there.
//
// What differs is the tile pipeline.  Because the PV product of tile k runs during step k+1,
// V tile k is only needed one step after K tile k, so it is also fetched one step later:
// step k reads K(k) and V(k-1) while K(k+1) and V(k) arrive.  Two K and two V buffers
// (64 KB) then suffice where fetching K and V together needs a third V buffer, and with
// 4 wavefronts of under 256 registers two workgroups share a CU: their barriers are
// independent and one's prologue (Q gather, 2 KB of state per row), stop/drain tail and
// epilogue overlap the other's tiles.
#include "s2o_internal.h"

namespace s2o {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) i16x4 lds_i16x4;
typedef __attribute__((address_space(1))) void gvoid;
typedef __attribute__((address_space(3))) void lvoid;

constexpr int kD = 128, kBN = 64;
constexpr int kWaves = 4, kThreads = 64 * kWaves, kRowsPerWave = 32;
constexpr int kRowElems = kD;
constexpr int kTileElems = kBN * kRowElems;
constexpr size_t kPrefixLds = (size_t)(4 * kTileElems) * 2 + 64;   // K x2, V x2, vote flags

__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 t = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, t);
}

// kNoStop: stop_mode 2 (every prefix tile folded in, the paper's kernel C) as an instantiation
// of its own, so that neither loop's registers weigh on the other.
template <bool kNoStop>
__global__ __launch_bounds__(kThreads, 2) void s2o_prefix_kernel(const AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* Ks = reinterpret_cast<uint16_t*>(smem);
  uint16_t* Vt = Ks + 2 * kTileElems;
  int* sflag = reinterpret_cast<int*>(Vt + 2 * kTileElems);   // stop votes: two sets of kWaves

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m_ = lane & 31, hh = lane >> 5;
  const int G = a.H / a.Hkv;
  const int BM = a.BM;                                   // query tile rows: 64 or 128
  const int wpt = BM / kRowsPerWave;                     // wavefronts per query tile
  const int tpw = kWaves / wpt;                          // query tiles per workgroup
  const int TJ = a.S / BM;                               // query tiles per segment
  const int JG = (TJ + tpw - 1) / tpw;                   // workgroups per (z,h,n)

  // ---- block -> (z, h, n, jg).  Longest prefixes first.  Consecutive block ids are dealt
  // round-robin to the 8 XCDs, each with its own L2: the JG workgroups of one (z, h, n) walk
  // the same KV_perm row at about the same time, so they are given ids that land on one XCD
  // (their gathered K/V tiles then hit in that L2), while the XCD of a head rotates with the
  // segment so that heads that stop early and heads that never stop mix evenly on every XCD.
  int z, h, n, jg;
  {
    const int ZH = a.Z * a.H;
    const int b = blockIdx.x;
    int zh_, nr;
    if (ZH % 8 == 0) {
      const int xcd = b & 7, idx = b >> 3, per = ZH / 8;
      jg = idx % JG;
      const int unit = idx / JG;
      nr = unit / per;
      zh_ = ((xcd - nr) & 7) + 8 * (unit % per);
    } else {
      jg = b % JG;
      const int unit = b / JG;
      nr = unit / ZH;
      zh_ = unit % ZH;
    }
    n = a.N - 1 - nr;
    z = zh_ / a.H;
    h = zh_ % a.H;
  }
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
  const int ntiles = a.max_tiles > 0 ? min(nK_all, a.max_tiles) : nK_all;

  // wavefront -> (query tile of the workgroup, 32-row part); the parts of a tile are
  // wavefronts tile, tile + tpw, ...
  const int tile_l = wave % tpw, part = wave / tpw;
  const int j = jg * tpw + tile_l;              // this wavefront's permuted query tile
  const bool active = j < TJ;

  // ---- loader: every wavefront moves 16 rows of K and 16 rows of V per step, 4 rows per
  // instruction (lane l: one 16-byte chunk of row 4*group + l/16, straight into LDS).  The
  // token indices are read two tiles ahead of the K fetch that uses them, so a fetch never
  // waits for its own index loads; the V fetch of a tile reuses its K fetch's indices.
  auto swz = [](int r) { return ((r & 3) << 2) | (((r >> 2) & 1) << 1) | ((r >> 3) & 1); };
  const uint32_t k_stride_bytes = (uint32_t)(a.ks[2] * 2), v_stride_bytes = (uint32_t)(a.vs[2] * 2);
  int goff[4];
#pragma unroll
  for (int gi = 0; gi < 4; ++gi) goff[gi] = 16 * ((lane & 15) ^ swz(16 * wave + 4 * gi + (lane >> 4)));
  uint32_t tokk[4], tokv[4];            // tokens of the next K tile and of the next V tile
  auto load_index = [&](int t) {        // tokk <- tile t (clamped); only called when ntiles > 0
    const int pt = min(t, ntiles - 1);
#pragma unroll
    for (int gi = 0; gi < 4; ++gi) {
      const int tk = kvrow[(int64_t)pt * kBN + 16 * wave + 4 * gi + (lane >> 4)];
      tokk[gi] = (uint32_t)min(max(tk, 0), a.L - 1);
    }
  };
  auto load_k = [&](int t) {            // K tile t (its tokens are in tokk) -> buffer t & 1
    uint16_t* kd = Ks + (t & 1) * kTileElems;
#pragma unroll
    for (int gi = 0; gi < 4; ++gi) {
      const char* kp = reinterpret_cast<const char*>(Kh) + (uint64_t)tokk[gi] * k_stride_bytes + goff[gi];
      __builtin_amdgcn_global_load_lds((const gvoid*)kp, (lvoid*)(kd + (16 * wave + 4 * gi) * kRowElems), 16, 0, 0);
    }
  };
  auto load_v = [&](int t) {            // V tile t (its tokens are in tokv) -> buffer t & 1
    uint16_t* vd = Vt + (t & 1) * kTileElems;
#pragma unroll
    for (int gi = 0; gi < 4; ++gi) {
      const char* vp = reinterpret_cast<const char*>(Vh) + (uint64_t)tokv[gi] * v_stride_bytes + goff[gi];
      __builtin_amdgcn_global_load_lds((const gvoid*)vp, (lvoid*)(vd + (16 * wave + 4 * gi) * kRowElems), 16, 0, 0);
    }
  };
  // the fetches of step t: K(t+1) and V(t); afterwards tokk holds tile t+2, tokv tile t+1
  auto load_step = [&](int t) {
    if (t + 1 < ntiles) load_k(t + 1);
    load_v(t);
#pragma unroll
    for (int gi = 0; gi < 4; ++gi) tokv[gi] = tokk[gi];
    load_index(t + 2);
  };
  constexpr bool no_stop = kNoStop;        // no stop rule: PV follows its scores at once, V comes with K
  if (ntiles > 0) {
    load_index(0);
    load_k(0);
#pragma unroll
    for (int gi = 0; gi < 4; ++gi) tokv[gi] = tokk[gi];
    if (no_stop) load_v(0);
    load_index(1);
  }

  // ---- the query row of this lane and its Q fragments
  int qoff;
  bf16x8 qf[8];
  {
    const int r = min(j, TJ - 1) * BM + kRowsPerWave * part + m_;
    qoff = a.use_q_perm ? a.q_perm[(zh * a.N + n) * a.S + r] : r;
    qoff = min(max(qoff, 0), a.S - 1);
    const uint16_t* qrow = Qh + (int64_t)(nS + qoff) * a.qs[2];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
      qf[kk] = *reinterpret_cast<const bf16x8*>(qrow + 16 * kk + 8 * hh);
  }

  // K operand: row 32*nb + m_, chunk 2*kk + hh -> per-lane byte offsets for the 8 steps
  int koff[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) koff[kk] = m_ * kRowElems + 8 * ((2 * kk + hh) ^ swz(m_));
  // transposing read of 4 keys x this lane's dimension (see attention.hip)
  int voff[4][2];
  {
    const int rl = ((lane & 15) >> 2) + 4 * (lane >> 5);
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int a8 = 0; a8 < 2; ++a8) {
        const int chunk = 4 * db + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
        voff[db][a8] = (rl + 8 * a8) * kRowElems + 8 * (chunk ^ swz(rl + 8 * a8)) + 4 * (lane & 1);
      }
  }
  auto read_vt = [&](const uint16_t* vt, int key0, int db) -> bf16x8 {
    const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(vt + key0 * kRowElems + voff[db][0]));
    const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(vt + key0 * kRowElems + voff[db][1]));
    u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
    u32x4 w = {l2.x, l2.y, h2.x, h2.y};
    return __builtin_bit_cast(bf16x8, w);
  };

  // ---- online-softmax state and output accumulator O^T[d-block], resumed from the state
  // buffers: row (z, h, l) -> acc [128] fp32 in the accumulator's register order, l, m.  The
  // statistics are needed by the first softmax; the accumulator only by the first PV product,
  // one step later: its 512 bytes per row are requested after the first tile's scores have
  // been issued and arrive behind them.
  constexpr float kLazy = 8.0f;
  const float c2 = a.scale_log2e;
  const int64_t st_row = zh * a.L + nS + qoff;
  float m_ref = a.st_m[st_row], l_run = a.st_l[st_row];
  f32x16 o[4];
  auto load_acc = [&] {
    const float* sp = a.st_acc + st_row * kD + 64 * hh;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(sp + 16 * db + 4 * i4);
        o[db][4 * i4] = v[0]; o[db][4 * i4 + 1] = v[1]; o[db][4 * i4 + 2] = v[2]; o[db][4 * i4 + 3] = v[3];
      }
  };
  int committed = 0, issued = 0;

  // values a tile's score step hands to its PV step
  f32x16 s[2];
  float alpha, mass, prev, m_use;
  bool grow;

  // S^T = K Q^T for key tile buffer kbuf
  auto qk = [&](int kbuf) {
    const uint16_t* ks = Ks + kbuf * kTileElems;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int i = 0; i < 16; ++i) s[nb][i] = 0.f;
    // K fragments are fetched from LDS two contraction steps ahead of the MFMA that uses them
    bf16x8 ka[3][2];
#pragma unroll
    for (int pre = 0; pre < 2; ++pre)
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
        ka[pre][nb] = *reinterpret_cast<const bf16x8*>(ks + 32 * nb * kRowElems + koff[pre]);
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      if (kk + 2 < 8) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
          ka[(kk + 2) % 3][nb] = *reinterpret_cast<const bf16x8*>(ks + 32 * nb * kRowElems + koff[kk + 2]);
      }
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
        s[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kk % 3][nb], qf[kk], s[nb], 0, 0, 0);
    }
  };
  // softmax numerators (left in s) and the row statistics of the tile
  auto softmax = [&] {
    float mx = -INFINITY;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[nb][i]);
    mx = fmaxf(mx, __shfl_xor(mx, 32)) * c2;
    grow = mx > m_ref + kLazy;
    m_use = grow ? mx : m_ref;
    float sum = 0.f;
    const float neg = -m_use;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float pe = __builtin_amdgcn_exp2f(fmaf(s[nb][i], c2, neg));
        s[nb][i] = pe;
        sum += pe;
      }
    sum += __shfl_xor(sum, 32);
    mass = sum;
    alpha = grow ? __builtin_amdgcn_exp2f(m_ref - m_use) : 1.0f;
    prev = l_run * alpha;
  };
  // rare: move the accumulator to a new reference maximum (O^T *= alpha)
  auto rescale = [&](float al, bool gr) {
    if (__builtin_amdgcn_ballot_w64(gr) != 0ull) {
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] *= al;
    }
  };
  // O^T += V^T P^T with the V tile in buffer vbuf
  auto pv = [&](int vbuf, const bf16x8 (&pb)[4]) {
    const uint16_t* vt = Vt + vbuf * kTileElems;
    // V^T fragments are fetched one contraction step (4 blocks of 32 dims) ahead
    bf16x8 va[2][4];
#pragma unroll
    for (int db = 0; db < 4; ++db) va[0][db] = read_vt(vt, 0, db);
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      if (st + 1 < 4) {
#pragma unroll
        for (int db = 0; db < 4; ++db) va[(st + 1) & 1][db] = read_vt(vt, 16 * (st + 1), db);
      }
#pragma unroll
      for (int db = 0; db < 4; ++db)
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[st & 1][db], pb[st], o[db], 0, 0, 0);
    }
  };

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
  auto pack_p = [&] {                   // P^T fragments (bf16) for the four 16-key contraction steps
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      const int nb = st >> 1, k2 = st & 1;
      u32x4 w;
#pragma unroll
      for (int q = 0; q < 4; ++q)
        w[q] = pack_bf16x2(s[nb][8 * k2 + 2 * q], s[nb][8 * k2 + 2 * q + 1]);
      pb_pend[st] = __builtin_bit_cast(bf16x8, w);
    }
  };
  auto vote_flags = [&](int step) { return sflag + kWaves * (step & 1); };
  auto publish = [&](int step) {        // after softmax of tile `step`: vote + speculative stats
    const bool keep = __builtin_amdgcn_ballot_w64(mass >= a.tau * prev) != 0ull;
    if (lane == 0) vote_flags(step)[wave] = keep ? 1 : 0;
    l_save = l_run; m_save = m_ref;
    l_run = prev + mass; m_ref = m_use;
    alpha_pend = alpha; grow_pend = grow;
    pack_p();
    ++issued;
  };
  auto tile_votes = [&](const int* vf) {
    int votes = 0;
    for (int p2 = 0; p2 < wpt; ++p2) votes |= vf[tile_l + tpw * p2];
    return votes;
  };
  auto wg_votes = [&](const int* vf) {
    int any = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) any |= vf[w];
    return any;
  };

  bool acc_loaded = false;
  if (no_stop && ntiles > 0) {
    // ---- every prefix tile is folded in (no votes, nothing deferred): step k reads K(k) and
    // V(k) while K(k+1) and V(k+1) arrive
    __syncthreads();                            // K and V tile 0 have landed
    for (int it = 0; it < ntiles; ++it) {
      if (it + 1 < ntiles) {
        load_k(it + 1);
#pragma unroll
        for (int gi = 0; gi < 4; ++gi) tokv[gi] = tokk[gi];
        load_v(it + 1);
        load_index(it + 2);
      }
      if (active) {
        qk(it & 1);
        if (!acc_loaded) { load_acc(); acc_loaded = true; }
        softmax();
        pack_p();
        rescale(alpha, grow);
        pv(it & 1, pb_pend);
        l_run = prev + mass; m_ref = m_use;
        ++committed; ++issued;
      }
      __syncthreads();
    }
  } else if (ntiles > 0) {
    __syncthreads();                            // K tile 0 has landed
    int it = 0;
    bool wg_done = false;
    if (active) {
      // first tile: scores only
      load_step(0);
      qk(0);
      load_acc(); acc_loaded = true;
      softmax();
      publish(0);
      __syncthreads();
      bool pending = true;                      // a scored tile waits for its vote
      for (it = 1; it < ntiles; ++it) {
        const int* vf = vote_flags(it - 1);
        const int votes = tile_votes(vf);
        if (votes == 0) {
          const int any = wg_votes(vf);
          if (a.stop_mode == 0) {
            l_run = l_save; m_ref = m_save;
          } else {
            rescale(alpha_pend, grow_pend);
            pv((it - 1) & 1, pb_pend);
            ++committed;
          }
          pending = false;
          wg_done = any == 0;
          break;
        }
        qk(it & 1);
        load_step(it);
        rescale(alpha_pend, grow_pend);
        pv((it - 1) & 1, pb_pend);
        ++committed;
        softmax();
        publish(it);
        __syncthreads();
      }
      if (pending) {                            // the last tile: its vote is visible now
        const bool stop = tile_votes(vote_flags(ntiles - 1)) == 0;
        if (stop && a.stop_mode == 0) {
          l_run = l_save; m_ref = m_save;
        } else {
          rescale(alpha_pend, grow_pend);
          pv((ntiles - 1) & 1, pb_pend);
          ++committed;
        }
        wg_done = true;
      }
    }
    // ---- drain: keep the tile pipeline fed until every query tile of the workgroup has stopped
    if (!wg_done) {
      for (; it < ntiles; ++it) {
        if (it > 0 && wg_votes(vote_flags(it - 1)) == 0) break;
        load_step(it);
        if (lane == 0) vote_flags(it)[wave] = 0;
        __syncthreads();
      }
    }
  }

  if (active) {
    if (!acc_loaded) load_acc();                 // no prefix tile was walked (first segment)
    // normalise and scatter to the original row: lane holds dims 32*db + 8*(i/4) + 4*hh + i%4
    const float inv = 1.0f / l_run;
    uint16_t* orow = Oh + (int64_t)(nS + qoff) * a.os[2];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        u32x2 w;
        w.x = pack_bf16x2(o[db][4 * i4] * inv, o[db][4 * i4 + 1] * inv);
        w.y = pack_bf16x2(o[db][4 * i4 + 2] * inv, o[db][4 * i4 + 3] * inv);
        *reinterpret_cast<u32x2*>(orow + 32 * db + 8 * i4 + 4 * hh) = w;
      }
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
    const void* fns[2] = {reinterpret_cast<const void*>(&s2o_prefix_kernel<false>),
                          reinterpret_cast<const void*>(&s2o_prefix_kernel<true>)};
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
  if (a.stop_mode == 2)
    hipLaunchKernelGGL(s2o_prefix_kernel<true>, dim3((unsigned)blocks), dim3(kThreads), kPrefixLds, stream, a);
  else
    hipLaunchKernelGGL(s2o_prefix_kernel<false>, dim3((unsigned)blocks), dim3(kThreads), kPrefixLds, stream, a);
  return hipGetLastError();
}

}  // namespace s2o
