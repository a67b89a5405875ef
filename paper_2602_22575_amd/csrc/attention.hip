// S2O sparse attention for gfx950 (paper Sec. 3.2-3.3; Alg. 2 + Alg. 3, Alg. 4 when the
// query order is the identity).
//
// One workgroup = 4 wavefronts = 4 permuted query tiles (4 x 64 rows) of one
// (batch, head, segment).  All query tiles of a segment walk the same KV_perm row, so the
// workgroup stages each gathered 64-token K/V tile in LDS once and the four wavefronts share
// it; every wavefront owns one query tile, keeps its Q fragments, online-softmax state and
// output accumulator in registers, and takes the early-stop branch on its own (the stop
// decision is uniform per wavefront).  The dense intra-segment causal window (Pass-1) is
// run by the same loop before the prefix walk, with identity indices and a per-element
// causal mask, so its state never leaves registers.
//
// MFMA formulation (v_mfma_f32_32x32x16_bf16), transposed so that a query row lives in
// one lane pair and softmax statistics need a single cross-lane step:
//   S^T[n, m] = sum_d K[n, d] Q[m, d]        A = K tile rows from LDS, B = Q from registers
//   O^T[d, m] = sum_n V^T[d, n] P^T[n, m]    A = V^T from LDS,        B = P from the S^T
//                                            accumulators (no data movement)
// Lane l = (m = l % 32, hh = l / 32).  A 32x32 accumulator block holds, in register i of lane
// l, the element [row 8*(i/4) + 4*hh + i%4][column m].  The B operand of the PV product takes
// registers 8*kk..8*kk+7 of an S^T block as its 8 contraction slots, so slot (hh, jj) is key
// 16*kk + 8*(jj/4) + 4*hh + jj%4 of the 32-key block; V^T is stored in LDS with the keys of
// each 16-group permuted accordingly (position 8*hh + 4*a + j holds key 8*a + 4*hh + j), which
// makes both LDS operand reads plain 16-byte loads.
#include "s2o_internal.h"

namespace s2o {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kD = 128;          // head dim
constexpr int kBN = 64;          // key tile
constexpr int kBM = 64;          // query tile (one wavefront)
constexpr int kWaves = 4;
constexpr int kKsStride = 136;   // bf16 elements per K row in LDS (272 B: conflict-free 16 B reads)
constexpr int kVtStride = 72;    // bf16 elements per V^T row in LDS (144 B)
constexpr int kKsElems = kBN * kKsStride;
constexpr int kVtElems = kD * kVtStride;
constexpr size_t kAttnLds = (size_t)(2 * kKsElems + 2 * kVtElems) * 2 + 64;

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

__global__ __launch_bounds__(256, 1) void s2o_attention_kernel(const AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* Ks = reinterpret_cast<uint16_t*>(smem);
  uint16_t* Vt = Ks + 2 * kKsElems;
  int* sflag = reinterpret_cast<int*>(Vt + 2 * kVtElems);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m_ = lane & 31, hh = lane >> 5;
  const int G = a.H / a.Hkv;
  const int TJ = a.S / kBM;                    // query tiles per segment
  const int JG = (TJ + kWaves - 1) / kWaves;   // workgroups per (z,h,n)

  // ---- block -> (z, h, n, jg).  Longest prefixes first; when the number of (z, KV head)
  // pairs is a multiple of 8, consecutive block ids (which the dispatcher deals round-robin
  // to the 8 XCDs) are mapped so that all work on one KV head stays on one XCD's L2.
  int z, h, n, jg;
  {
    const int U = a.Z * a.Hkv;
    int b = blockIdx.x, unit, rest;
    if (U % 8 == 0) {
      const int xcd = b & 7, idx = b >> 3, per = U / 8;
      unit = (idx % per) * 8 + xcd;
      rest = idx / per;
    } else {
      unit = b % U;
      rest = b / U;
    }
    jg = rest % JG; rest /= JG;
    const int hq = rest % G; rest /= G;
    n = a.N - 1 - rest;
    z = unit / a.Hkv;
    const int g = unit % a.Hkv;
    h = g * G + hq;
  }
  const int g = h / G;
  const uint16_t* Qh = a.Q + z * a.qs[0] + h * a.qs[1];
  const uint16_t* Kh = a.K + z * a.ks[0] + g * a.ks[1];
  const uint16_t* Vh = a.V + z * a.vs[0] + g * a.vs[1];
  uint16_t* Oh = a.O + z * a.os[0] + h * a.os[1];
  const int64_t zh = (int64_t)z * a.H + h;
  const int32_t* kvrow = a.kv_perm + zh * kv_row_offset(a.N, a.S) + kv_row_offset(n, a.S);
  const int nS = n * a.S;
  const int nK = nS / kBN;                     // prefix tiles of this segment

  const int j = jg * kWaves + wave;            // this wavefront's permuted query tile
  bool active = j < TJ;

  // ---- query rows of this lane (two: mb = 0, 1) and their Q fragments
  int qoff[2];
  bf16x8 qf[2][8];
#pragma unroll
  for (int mb = 0; mb < 2; ++mb) {
    const int r = min(j, TJ - 1) * kBM + 32 * mb + m_;
    qoff[mb] = a.use_q_perm ? a.q_perm[(zh * a.N + n) * a.S + r] : r;
    qoff[mb] = min(max(qoff[mb], 0), a.S - 1);
    const uint16_t* qrow = Qh + (int64_t)(nS + qoff[mb]) * a.qs[2];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
      qf[mb][kk] = *reinterpret_cast<const bf16x8*>(qrow + 16 * kk + 8 * hh);
  }
  const int wave_pmax = active ? wave_max_i32(max(qoff[0], qoff[1])) : -1;
  if (lane == 0) sflag[wave] = wave_pmax;
  __syncthreads();
  const int wg_pmax = max(max(sflag[0], sflag[1]), max(sflag[2], sflag[3]));
  const int nloc = wg_pmax / kBN + 1;          // own-segment key tiles this workgroup needs
  const int ntiles = nloc + nK;
  __syncthreads();

  // ---- loader: thread (c, gq) moves 16-byte chunk c of key slots 4*gq .. 4*gq+3
  const int c = tid & 15, gq = tid >> 4;
  // V^T position of slot 4*gq: swap bits 0 and 1 of gq (see the header comment)
  const int vpos = 4 * ((gq & ~3) | ((gq & 1) << 1) | ((gq >> 1) & 1));
  u32x4 kreg[4], vreg[4];
  auto load_tile = [&](int it) {
    int tok[4];
    if (it < nloc) {
#pragma unroll
      for (int s = 0; s < 4; ++s) tok[s] = nS + it * kBN + 4 * gq + s;
    } else {
      const int4 t4 = *reinterpret_cast<const int4*>(kvrow + (int64_t)(it - nloc) * kBN + 4 * gq);
      tok[0] = t4.x; tok[1] = t4.y; tok[2] = t4.z; tok[3] = t4.w;
#pragma unroll
      for (int s = 0; s < 4; ++s) tok[s] = min(max(tok[s], 0), a.L - 1);
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      kreg[s] = *reinterpret_cast<const u32x4*>(Kh + (int64_t)tok[s] * a.ks[2] + 8 * c);
      vreg[s] = *reinterpret_cast<const u32x4*>(Vh + (int64_t)tok[s] * a.vs[2] + 8 * c);
    }
  };
  auto store_tile = [&](int buf) {
    uint16_t* ks = Ks + buf * kKsElems;
    uint16_t* vt = Vt + buf * kVtElems;
#pragma unroll
    for (int s = 0; s < 4; ++s)
      *reinterpret_cast<u32x4*>(ks + (4 * gq + s) * kKsStride + 8 * c) = kreg[s];
#pragma unroll
    for (int q = 0; q < 4; ++q) {   // dword q of a chunk holds dims 8c+2q (low half), 8c+2q+1
      u32x2 lo, hi;
      lo.x = (vreg[0][q] & 0xffffu) | (vreg[1][q] << 16);
      lo.y = (vreg[2][q] & 0xffffu) | (vreg[3][q] << 16);
      hi.x = (vreg[0][q] >> 16) | (vreg[1][q] & 0xffff0000u);
      hi.y = (vreg[2][q] >> 16) | (vreg[3][q] & 0xffff0000u);
      *reinterpret_cast<u32x2*>(vt + (8 * c + 2 * q) * kVtStride + vpos) = lo;
      *reinterpret_cast<u32x2*>(vt + (8 * c + 2 * q + 1) * kVtStride + vpos) = hi;
    }
  };

  // ---- online-softmax state (base-2 logits) and output accumulator O^T[d-block][mb]
  float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};
  f32x16 o[4][2];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[db][mb][i] = 0.f;
  int committed = 0, issued = 0;

  load_tile(0);
  store_tile(0);
  __syncthreads();

  for (int it = 0; it < ntiles; ++it) {
    const int buf = it & 1;
    if (it + 1 < ntiles) load_tile(it + 1);

    const bool local = it < nloc;
    if (active && !(local && it * kBN > wave_pmax)) {
      const uint16_t* ks = Ks + buf * kKsElems;
      const uint16_t* vt = Vt + buf * kVtElems;
      // S^T = K Q^T
      f32x16 s[2][2];
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int i = 0; i < 16; ++i) s[nb][mb][i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
          const bf16x8 ka = *reinterpret_cast<const bf16x8*>(ks + (32 * nb + m_) * kKsStride + 16 * kk + 8 * hh);
#pragma unroll
          for (int mb = 0; mb < 2; ++mb)
            s[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[mb][kk], s[nb][mb], 0, 0, 0);
        }
      }
      // online softmax per query row (= per lane and mb)
      float m_new[2], alpha[2], mass[2], prev[2];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        float mx = -INFINITY;
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            float x = s[nb][mb][i] * a.scale_log2e;
            if (local) {
              const int kpos = it * kBN + 32 * nb + 8 * (i >> 2) + 4 * hh + (i & 3);
              x = kpos > qoff[mb] ? -INFINITY : x;     // CausalMask
            }
            s[nb][mb][i] = x;
            mx = fmaxf(mx, x);
          }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        m_new[mb] = fmaxf(m_run[mb], mx);
        float sum = 0.f;
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const float p = __builtin_amdgcn_exp2f(s[nb][mb][i] - m_new[mb]);
            s[nb][mb][i] = p;
            sum += p;
          }
        sum += __shfl_xor(sum, 32);
        mass[mb] = sum;
        alpha[mb] = __builtin_amdgcn_exp2f(m_run[mb] - m_new[mb]);
        prev[mb] = l_run[mb] * alpha[mb];
      }
      bool stop = false;
      if (!local) {
        // early-stop rule: continue iff some row's tile mass reaches tau * (mass so far)
        const bool keep = (mass[0] >= a.tau * prev[0]) || (mass[1] >= a.tau * prev[1]);
        stop = __builtin_amdgcn_ballot_w64(keep) == 0ull;
        ++issued;
      }
      if (stop) active = false;
      if (!(stop && a.stop_mode == 0)) {
        if (!local) ++committed;
        bf16x8 pb[2][2][2];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
          l_run[mb] = prev[mb] + mass[mb];
          m_run[mb] = m_new[mb];
#pragma unroll
          for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[db][mb][i] *= alpha[mb];
#pragma unroll
          for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int k2 = 0; k2 < 2; ++k2) {
              u32x4 w;
#pragma unroll
              for (int q = 0; q < 4; ++q)
                w[q] = pack_bf16x2(s[nb][mb][8 * k2 + 2 * q], s[nb][mb][8 * k2 + 2 * q + 1]);
              pb[nb][mb][k2] = __builtin_bit_cast(bf16x8, w);
            }
        }
        // O^T += V^T P^T
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
          for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
            for (int db = 0; db < 4; ++db) {
              const bf16x8 va = *reinterpret_cast<const bf16x8*>(vt + (32 * db + m_) * kVtStride + 32 * nb + 16 * k2 + 8 * hh);
#pragma unroll
              for (int mb = 0; mb < 2; ++mb)
                o[db][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[nb][mb][k2], o[db][mb], 0, 0, 0);
            }
      }
    }

    if (it + 1 < ntiles) store_tile(buf ^ 1);
    if (lane == 0) sflag[wave] = active ? 1 : 0;
    __syncthreads();
    // once the prefix walk has begun, the workgroup leaves when every wavefront has stopped
    if (it + 1 >= nloc && (sflag[0] | sflag[1] | sflag[2] | sflag[3]) == 0) break;
    __syncthreads();
  }

  if (j < TJ) {
    // normalise and scatter to the original rows: lane holds, for row (mb, m), dims
    // 32*db + 8*(i/4) + 4*hh + i%4
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
      const float inv = 1.0f / l_run[mb];
      uint16_t* orow = Oh + (int64_t)(nS + qoff[mb]) * a.os[2];
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          u32x2 w;
          w.x = pack_bf16x2(o[db][mb][4 * i4] * inv, o[db][mb][4 * i4 + 1] * inv);
          w.y = pack_bf16x2(o[db][mb][4 * i4 + 2] * inv, o[db][mb][4 * i4 + 3] * inv);
          *reinterpret_cast<u32x2*>(orow + 32 * db + 8 * i4 + 4 * hh) = w;
        }
    }
    if (lane == 0) {
      const int64_t ci = zh * (a.L / kBM) + (int64_t)n * TJ + j;
      if (a.computed) a.computed[ci] = committed;
      if (a.skipped) a.skipped[ci] = nK - issued;
    }
  }
}

hipError_t launch_attention(const AttnArgs& a, hipStream_t stream) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&s2o_attention_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kAttnLds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int TJ = a.S / kBM;
  const int JG = (TJ + kWaves - 1) / kWaves;
  const int64_t blocks = (int64_t)a.Z * a.H * a.N * JG;
  if (blocks <= 0 || blocks > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(s2o_attention_kernel, dim3((unsigned)blocks), dim3(256), kAttnLds, stream, a);
  return hipGetLastError();
}

}  // namespace s2o
