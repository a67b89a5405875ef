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
// and prefix.hip, which share this file's formulation.)
//
// MFMA formulation (v_mfma_f32_32x32x16_bf16), transposed so that a query row lives in
// one lane pair and softmax statistics need a single cross-lane step:
//   S^T[n, m] = sum_d K[n, d] Q[m, d]        A = K tile rows from LDS, B = Q from registers
//   O^T[d, m] = sum_n V^T[d, n] P^T[n, m]    A = V^T from LDS,        B = P from the S^T
//                                            accumulators (no data movement)
// Lane l = (m = l % 32, hh = l / 32).  A 32x32 accumulator block holds, in register i of lane
// l, the element [row 8*(i/4) + 4*hh + i%4][column m].  The B operand of the PV product takes
// registers 8*kk..8*kk+7 of an S^T block as its 8 contraction slots, so slot (hh, jj) is key
// 16*kk + 8*(jj/4) + 4*hh + jj%4 of the 32-key block.  K and V tiles sit row-major (token
// rows) in LDS, written there directly by global_load_lds (no staging registers): a
// wavefront instruction deposits 4 gathered rows as 1 KB, lane l at byte 16*l, so rows
// cannot be padded; bank conflicts are avoided by an XOR swizzle instead (lane l fetches
// chunk (l%16) ^ swz(row) of its row, swz(r) = 4*(r%4) + 2*((r/4)%2) + (r/8)%2: the 16 rows
// a 16-byte K read touches land on 16 different chunks, and the 4 rows x 64 bytes that half
// a wavefront touches in a transposing V read land on the four 16-bank groups).
// The K operand is a plain 16-byte read of a row; the V^T operand is read
// with the transposing LDS load ds_read_b64_tr_b16: within each group of 16 lanes, lane i
// receives element (i % 4) of the four 8-byte rows pointed to by lanes i/4, 4 + i/4, 8 + i/4
// and 12 + i/4, so pointing lane r of a group at (key slot r/4, dims 4*(r%4)..+3) hands every
// lane the four keys of its contraction slots at its own head dimension.
#include <type_traits>

#include "s2o_internal.h"

namespace s2o {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kD = 128;          // head dim
constexpr int kBN = 64;          // key tile
constexpr int kRowsPerWave = 32; // query rows of one wavefront
constexpr int kWaves = 8;        // a query tile of B_M rows is B_M/32 wavefronts: 4 tiles of 64
                                 // rows or 2 tiles of 128 rows per workgroup
constexpr int kThreads = 64 * kWaves;
constexpr int kRowElems = kD;    // K and V rows sit unpadded in LDS (256 B); the sixteen 16-byte
                                 // chunks of row r are stored at slot (chunk ^ swz(r)) instead
constexpr int kKsElems = kBN * kRowElems;
constexpr int kVtElems = kBN * kRowElems;
constexpr size_t kAttnLds = (size_t)(2 * kKsElems + 3 * kVtElems) * 2 + 256;

__device__ inline int wave_max_i32(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = max(v, __shfl_xor(v, o));
  return v;
}

__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 t = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, t);
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
    const uint16_t* qrow = Qh + (int64_t)(nS + qoff) * a.qs[2];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
      qf[kk] = *reinterpret_cast<const bf16x8*>(qrow + 16 * kk + 8 * hh);
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

  // ---- loader: wavefronts 0-3 move K, 4-7 move V, 4 groups of 4 rows each per tile; in a
  // group lane l moves one 16-byte chunk of row 4*group + l/16 straight into LDS
  auto swz = [](int r) { return ((r & 3) << 2) | (((r >> 2) & 1) << 1) | ((r >> 3) & 1); };
  const bool loads_v = wave >= 4;
  const uint16_t* src = loads_v ? Vh : Kh;
  const int64_t src_stride = loads_v ? a.vs[2] : a.ks[2];
  typedef __attribute__((address_space(1))) void gvoid;
  typedef __attribute__((address_space(3))) void lvoid;
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
    gbase[gi] = reinterpret_cast<const char*>(src) + 16 * ((lane & 15) ^ swz(16 * (wave & 3) + 4 * gi + (lane >> 4)));
  auto load_tile = [&](int it) {       // K tiles alternate between 2 buffers, V tiles between 3
    uint16_t* dst = loads_v ? Vt + (it % 3) * kVtElems : Ks + (it & 1) * kKsElems;
#pragma unroll
    for (int gi = 0; gi < 4; ++gi) {
      const uint32_t tok = (uint32_t)min(max(tokn[gi], 0), a.L - 1);
      const char* gp = gbase[gi] + (uint64_t)tok * stride_bytes;   // one 64-bit multiply-add
      __builtin_amdgcn_global_load_lds((const gvoid*)gp, (lvoid*)(dst + (16 * (wave & 3) + 4 * gi) * kRowElems),
                                       16, 0, 0);
    }
    load_index(it + 1);
  };
  // K operand: row 32*nb + m_, chunk 2*kk + hh -> per-lane byte offsets for the 8 steps
  int koff[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) koff[kk] = m_ * kRowElems + 8 * ((2 * kk + hh) ^ swz(m_));
  // transposing read of 4 keys x this lane's dimension: lane (group g16 = lane/16, r = lane%16)
  // points at key slot r/4 (+ 4 for the upper lane half), dims 16*(g16&1) + 4*(r%4); the row's
  // swizzle depends on the lane and on which 8-key half (a) of the 16-key step is read
  typedef short i16x4 __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) i16x4 lds_i16x4;
  int voff[4][2];
  {
    const int rl = ((lane & 15) >> 2) + 4 * (lane >> 5);          // row inside the 8-key half
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int a8 = 0; a8 < 2; ++a8) {
        const int chunk = 4 * db + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
        voff[db][a8] = (rl + 8 * a8) * kRowElems + 8 * (chunk ^ swz(rl + 8 * a8)) + 4 * (lane & 1);
      }
  }
  auto read_vt = [&](const uint16_t* vt, int key0, int db) -> bf16x8 {
    // contraction slots (hh, jj): jj < 4 -> keys key0 + 4*hh + jj, jj >= 4 -> keys key0 + 8 + 4*hh + jj - 4
    const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(vt + key0 * kRowElems + voff[db][0]));
    const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(vt + key0 * kRowElems + voff[db][1]));
    u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
    u32x4 w = {l2.x, l2.y, h2.x, h2.y};
    return __builtin_bit_cast(bf16x8, w);
  };

  // ---- online-softmax state and output accumulator O^T[d-block].  Logits are kept in
  // base-2 units (raw score * softmax_scale * log2 e).  m_ref is the reference maximum the
  // accumulated terms are expressed in; it follows the true running maximum lazily: terms
  // are only rescaled when the maximum has grown by more than kLazy (2^8), so that in the
  // common case a tile costs no pass over the accumulator.  Any reference gives the same
  // result; tile masses and the stop test are ratios in one common reference.
  constexpr float kLazy = 8.0f;
  float m_ref = -INFINITY, l_run = 0.f;
  f32x16 o[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
  int committed = 0, issued = 0;
  const float c2 = a.scale_log2e;

  // values a tile's score step hands to its PV step
  f32x16 s[2];
  float alpha, mass, prev, m_use;
  bool grow;

  // S^T = K Q^T for key tile buffer kbuf
  auto qk = [&](int kbuf) {
    const uint16_t* ks = Ks + kbuf * kKsElems;
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
  auto softmax = [&](auto local_tag, int it) {
    constexpr bool kLocal = decltype(local_tag)::value;
    float mx = -INFINITY;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        if (kLocal) {
          const int kpos = it * kBN + 32 * nb + 8 * (i >> 2) + 4 * hh + (i & 3);
          if (kpos > qoff) s[nb][i] = -INFINITY;     // CausalMask
        }
        mx = fmaxf(mx, s[nb][i]);
      }
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
  // P^T fragments (bf16) for the four 16-key contraction steps
  auto pack_p = [&](bf16x8 (&pb)[4]) {
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      const int nb = st >> 1, k2 = st & 1;
      u32x4 w;
#pragma unroll
      for (int q = 0; q < 4; ++q)
        w[q] = pack_bf16x2(s[nb][8 * k2 + 2 * q], s[nb][8 * k2 + 2 * q + 1]);
      pb[st] = __builtin_bit_cast(bf16x8, w);
    }
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
    const uint16_t* vt = Vt + vbuf * kVtElems;
    // V^T fragments are fetched one contraction step (4 blocks of 32 dims) ahead
    bf16x8 va[2][4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
      va[0][db] = read_vt(vt, 0, db);
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      if (st + 1 < 4) {
#pragma unroll
        for (int db = 0; db < 4; ++db)
          va[(st + 1) & 1][db] = read_vt(vt, 16 * (st + 1), db);
      }
#pragma unroll
      for (int db = 0; db < 4; ++db)
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[st & 1][db], pb[st], o[db], 0, 0, 0);
    }
  };

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
      if (!own) softmax(std::false_type{}, it);
      else softmax(std::true_type{}, it);
      bf16x8 pb[4];
      pack_p(pb);
      rescale(alpha, grow);
      pv(it % 3, pb);
      l_run = prev + mass;
      m_ref = m_use;
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
    const bool keep = __builtin_amdgcn_ballot_w64(mass >= a.tau * prev) != 0ull;
    if (lane == 0) vote_flags(step)[wave] = keep ? 1 : 0;
    l_save = l_run; m_save = m_ref;
    l_run = prev + mass; m_ref = m_use;
    alpha_pend = alpha; grow_pend = grow;
    pack_p(pb_pend);
    pending = true;
    ++issued;
  };
  bool wg_done = false;
  if (active && it < ntiles) {
    // first prefix tile: scores only
    if (it + 1 < ntiles) load_tile(it + 1);
    qk(it & 1);
    softmax(std::false_type{}, it);
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
          rescale(alpha_pend, grow_pend);
          pv((it - 1) % 3, pb_pend);
          ++committed;
        }
        pending = false;
        wg_done = any == 0;
        break;
      }
      if (it + 1 < ntiles) load_tile(it + 1);
      rescale(alpha_pend, grow_pend);
      pv((it - 1) % 3, pb_pend);
      ++committed;
      softmax(std::false_type{}, it);
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
        rescale(alpha_pend, grow_pend);
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
}

size_t attention_state_bytes(int Z, int H, int L) {
  return (size_t)Z * H * L * (kD + 2) * sizeof(float);
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
