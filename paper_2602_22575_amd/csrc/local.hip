// S2O own-segment pass (paper Sec. 3.2, Alg. 2) for gfx950: dense causal attention of every
// query over the keys of its own segment, queries in original order, leaving the
// un-normalised online-softmax state (accumulator, l, m) per row for the prefix walk.
//
// One workgroup = 4 wavefronts = 128 consecutive query rows of one (batch, head, segment),
// 32 rows per wavefront; it needs the key tiles 0 .. (its last row) / 64 of the segment and
// the causal mask only where a row ends inside a tile.  Nothing here depends on the query
// tile size or on the index maps.  With K and V double-buffered a workgroup takes 64 KB of
// LDS and 4 wavefronts of under 256 registers, so two workgroups share a CU: their
// barriers are independent, and one's prologue (Q rows, first tile) and epilogue (2 KB of
// state per row) overlap the other's tiles -- with the 8-wavefront, one-workgroup-per-CU
// form of attention.hip those phases were exposed 64 times per CU.
//
// Tile pipeline, MFMA formulation, LDS layouts and the base-2 online softmax with lazy
// rescaling are those of attention.hip; see there.  The state layout (accumulator in the
// MFMA register order: a lane's 16 values of a 32-dim block contiguous) is shared with it.
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
constexpr int kRowsPerWg = kWaves * kRowsPerWave;
constexpr int kRowElems = kD;
constexpr int kTileElems = kBN * kRowElems;
constexpr size_t kLocalLds = (size_t)(4 * kTileElems) * 2;   // K x2, V x2

__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 t = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, t);
}

__global__ __launch_bounds__(kThreads, 2) void s2o_local_kernel(const AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* Ks = reinterpret_cast<uint16_t*>(smem);
  uint16_t* Vt = Ks + 2 * kTileElems;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m_ = lane & 31, hh = lane >> 5;
  const int G = a.H / a.Hkv;
  const int JG = (a.S + kRowsPerWg - 1) / kRowsPerWg;   // workgroups per (z,h,n)

  // ---- block -> (z, h, n, jg); a segment's workgroups on one XCD (they read the same K/V),
  // heads rotated over the XCDs per segment as in the prefix walk
  int z, h, n, jg;
  {
    const int ZH = a.Z * a.H;
    const int b = blockIdx.x;
    int zh_, nr;
    if (ZH % 8 == 0) {
      const int xcd = b & 7, idx = b >> 3, per = ZH / 8;
      jg = JG - 1 - idx % JG;                   // the longest workgroups of a segment first
      const int unit = idx / JG;
      nr = unit / per;
      zh_ = ((xcd - nr) & 7) + 8 * (unit % per);
    } else {
      jg = JG - 1 - b % JG;
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
  const int64_t zh = (int64_t)z * a.H + h;
  const int nS = n * a.S;

  // rows of this wavefront: r0 .. r0 + 31 (original order), all inside the segment or none
  const int r0 = jg * kRowsPerWg + kRowsPerWave * wave;
  const bool active = r0 < a.S;                 // S is a multiple of 64, r0 of 32
  const int qoff = min(r0 + m_, a.S - 1);
  const int wave_pmax = active ? min(r0 + kRowsPerWave - 1, a.S - 1) : -1;
  const int wg_pmax = min(jg * kRowsPerWg + kRowsPerWg, a.S) - 1;
  const int nloc = wg_pmax / kBN + 1;           // key tiles this workgroup needs
  const int myn = active ? wave_pmax / kBN + 1 : 0;   // ... and this wavefront

  // ---- loader: every wavefront moves 16 rows of K and 16 rows of V per tile, 4 rows per
  // instruction (lane l: one 16-byte chunk of row 4*group + l/16, straight into LDS)
  auto swz = [](int r) { return ((r & 3) << 2) | (((r >> 2) & 1) << 1) | ((r >> 3) & 1); };
  const uint32_t k_stride_bytes = (uint32_t)(a.ks[2] * 2), v_stride_bytes = (uint32_t)(a.vs[2] * 2);
  int goff[4];
#pragma unroll
  for (int gi = 0; gi < 4; ++gi) goff[gi] = 16 * ((lane & 15) ^ swz(16 * wave + 4 * gi + (lane >> 4)));
  auto load_tile = [&](int it) {
    uint16_t* kd = Ks + (it & 1) * kTileElems;
    uint16_t* vd = Vt + (it & 1) * kTileElems;
#pragma unroll
    for (int gi = 0; gi < 4; ++gi) {
      const uint32_t tok = (uint32_t)min(nS + it * kBN + 16 * wave + 4 * gi + (lane >> 4), a.L - 1);
      const char* kp = reinterpret_cast<const char*>(Kh) + (uint64_t)tok * k_stride_bytes + goff[gi];
      const char* vp = reinterpret_cast<const char*>(Vh) + (uint64_t)tok * v_stride_bytes + goff[gi];
      __builtin_amdgcn_global_load_lds((const gvoid*)kp, (lvoid*)(kd + (16 * wave + 4 * gi) * kRowElems), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((const gvoid*)vp, (lvoid*)(vd + (16 * wave + 4 * gi) * kRowElems), 16, 0, 0);
    }
  };
  load_tile(0);

  // ---- Q fragments of this lane's row
  bf16x8 qf[8];
  {
    const uint16_t* qrow = Qh + (int64_t)(nS + qoff) * a.qs[2];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
      qf[kk] = *reinterpret_cast<const bf16x8*>(qrow + 16 * kk + 8 * hh);
  }

  int koff[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) koff[kk] = m_ * kRowElems + 8 * ((2 * kk + hh) ^ swz(m_));
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

  constexpr float kLazy = 8.0f;
  const float c2 = a.scale_log2e;
  float m_ref = -INFINITY, l_run = 0.f;
  f32x16 o[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
  f32x16 s[2];

  __syncthreads();                              // tile 0 has landed

  for (int it = 0; it < nloc; ++it) {
    if (it + 1 < nloc) load_tile(it + 1);
    if (it < myn) {
      // ---- S^T = K Q^T
      const uint16_t* ks = Ks + (it & 1) * kTileElems;
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int i = 0; i < 16; ++i) s[nb][i] = 0.f;
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
      // ---- CausalMask (only if some row of the wavefront ends inside this tile), row maximum
      const bool masked = it * kBN + kBN - 1 > r0;
      float mx = -INFINITY;
      if (masked) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int kpos = it * kBN + 32 * nb + 8 * (i >> 2) + 4 * hh + (i & 3);
            if (kpos > qoff) s[nb][i] = -INFINITY;
            mx = fmaxf(mx, s[nb][i]);
          }
      } else {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
          for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[nb][i]);
      }
      mx = fmaxf(mx, __shfl_xor(mx, 32)) * c2;
      const bool grow = mx > m_ref + kLazy;
      const float m_use = grow ? mx : m_ref;
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
      const float alpha = grow ? __builtin_amdgcn_exp2f(m_ref - m_use) : 1.0f;
      // ---- P^T fragments, rare rescale, O^T += V^T P^T
      bf16x8 pb[4];
#pragma unroll
      for (int st = 0; st < 4; ++st) {
        const int nb = st >> 1, k2 = st & 1;
        u32x4 w;
#pragma unroll
        for (int q = 0; q < 4; ++q)
          w[q] = pack_bf16x2(s[nb][8 * k2 + 2 * q], s[nb][8 * k2 + 2 * q + 1]);
        pb[st] = __builtin_bit_cast(bf16x8, w);
      }
      if (__builtin_amdgcn_ballot_w64(grow) != 0ull) {
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
      }
      const uint16_t* vt = Vt + (it & 1) * kTileElems;
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
      l_run = l_run * alpha + sum;
      m_ref = m_use;
    }
    __syncthreads();
  }

  if (active) {
    // leave the un-normalised state for the prefix walk
    const int64_t st_row = zh * a.L + nS + qoff;
    float* sp = a.st_acc + st_row * kD + 64 * hh;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const f32x4 v = {o[db][4 * i4], o[db][4 * i4 + 1], o[db][4 * i4 + 2], o[db][4 * i4 + 3]};
        *reinterpret_cast<f32x4*>(sp + 16 * db + 4 * i4) = v;
      }
    if (hh == 0) { a.st_l[st_row] = l_run; a.st_m[st_row] = m_ref; }
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
  const int64_t blocks = (int64_t)a.Z * a.H * a.N * JG;
  if (blocks <= 0 || blocks > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(s2o_local_kernel, dim3((unsigned)blocks), dim3(kThreads), kLocalLds, stream, a);
  return hipGetLastError();
}

}  // namespace s2o
