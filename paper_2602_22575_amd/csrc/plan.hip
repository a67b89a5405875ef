// S2O ranking stage for gfx950 (paper Sec. 3.1, Alg. 1, Eqs. (1)-(2)).
//
//   kguide_kernel        k_guide = mean of the first key segment (k_mean[0]).
//   pool_sq_sort_kernel  one workgroup per (z, h, segment): a single pass over the
//                        segment's Q rows gives q_mean and s_Q; the S scores are then
//                        Argsort-ed in LDS (bitonic network on 64-bit keys) -> Q_perm.
//   score_kernel<MODE>   s_K[n, t] = <q_mean[n], K[t]> as an MFMA contraction per KV head:
//                        rows = (query head of the group, segment), columns = key tokens.
//                        q_mean is split exactly into three bf16 terms so that bf16 MFMA
//                        reproduces the fp32 x bf16 products exactly (fp32 accumulation).
//                        The kernel is run three times with different epilogues:
//                        MODE 0 row min/max (+ optional s_K store), MODE 1 bucket
//                        histogram, MODE 2 scatter of (key, token) pairs into buckets.
//   scan_kernel          per prefix row: bucket offsets and a list of spans (runs of
//                        consecutive buckets that fit the LDS sort).
//   span_sort_kernel     sorts each span in LDS and writes the token indices at their
//                        final ranks -> KV_perm.
//   big_sort_kernel      fallback for a bucket that alone exceeds the LDS sort (e.g. all
//                        scores equal): a stable LSD radix sort by one workgroup.
//
// Argsort semantics: descending score, ties by ascending index, -0 == +0.  Both sorts work
// on the 64-bit key (~ordered(score)) << 32 | index, whose ascending order is exactly
// that order, so no stability property of the network is needed.
#include "s2o_internal.h"

namespace s2o {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kD = 128;
constexpr int kNBMax = 512;        // buckets per prefix row (upper bound)
constexpr int kBucketAvg = 256;    // target average bucket population
constexpr int kSpanCap = 4096;     // elements one span_sort workgroup sorts in LDS
constexpr int kTokChunk = 1024;    // key tokens per score workgroup
constexpr int kBigGrid = 64;       // workgroups of the fallback sort

__host__ __device__ inline int row_buckets(int n, int S) {
  int64_t nb = (int64_t)n * S / kBucketAvg;
  return nb < 1 ? 1 : (nb > kNBMax ? kNBMax : (int)nb);
}

// float -> uint32 whose unsigned order is the float order (-0 canonicalised to +0)
__device__ inline uint32_t ordered_u32(float f) {
  uint32_t u = __float_as_uint(f);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ inline float ordered_to_float(uint32_t o) {
  return __uint_as_float((o & 0x80000000u) ? (o & 0x7fffffffu) : ~o);
}
__device__ inline uint64_t sort_key(float score, uint32_t idx) {
  return ((uint64_t)(~ordered_u32(score)) << 32) | idx;
}

__device__ inline float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// ---------------------------------------------------------------------------------------
struct Scratch {
  float* kguide;      // [Z*Hkv*128]
  float* qmean;       // [Z*H*N*128]
  uint16_t* qsplit;   // [Z*H*N][3][128] bf16
  uint32_t* rowmin;   // [Z*H*N] ordered-u32
  uint32_t* rowmax;   // [Z*H*N]
  uint32_t* hist;     // [Z*H*N*kNBMax]
  uint32_t* cursor;   // [Z*H*N*kNBMax]
  uint32_t* counters; // [0]=#spans [1]=#big spans [2]=error flag
  int4* spans;        // [max_spans]  (row, begin, end, 0)
  int4* bigspans;     // [max_spans]
  uint64_t* pairs;    // [Z*H*P]
  uint64_t* alt;      // [kBigGrid * L]
  int64_t max_spans;
  size_t total;
};

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static Scratch carve(void* base, int Z, int H, int Hkv, int L, int S) {
  const int64_t N = L / S;
  const int64_t rows = (int64_t)Z * H * N;
  const int64_t P = kv_row_offset(N, S);
  Scratch s;
  s.max_spans = (int64_t)Z * H * (3 * P / kSpanCap + 2 * N) + 8;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return (char*)base + o; };
  s.kguide = (float*)take((size_t)Z * Hkv * kD * 4);
  s.qmean = (float*)take((size_t)rows * kD * 4);
  s.qsplit = (uint16_t*)take((size_t)rows * 3 * kD * 2);
  s.rowmin = (uint32_t*)take((size_t)rows * 4);
  s.rowmax = (uint32_t*)take((size_t)rows * 4);
  s.hist = (uint32_t*)take((size_t)rows * kNBMax * 4);
  s.cursor = (uint32_t*)take((size_t)rows * kNBMax * 4);
  s.counters = (uint32_t*)take(64);
  s.spans = (int4*)take((size_t)s.max_spans * 16);
  s.bigspans = (int4*)take((size_t)s.max_spans * 16);
  s.pairs = (uint64_t*)take((size_t)Z * H * P * 8);
  s.alt = (uint64_t*)take((size_t)kBigGrid * L * 8);
  s.total = off;
  return s;
}

size_t plan_scratch_bytes(int Z, int H, int Hkv, int L, int S) {
  return carve(nullptr, Z, H, Hkv, L, S).total;
}

// ---------------------------------------------------------------------------------------
__global__ void init_kernel(Scratch s, int64_t rows) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < rows * kNBMax) s.hist[i] = 0;
  if (i < rows) { s.rowmin[i] = 0xffffffffu; s.rowmax[i] = 0u; }
  if (i < 16) s.counters[i] = 0;
}

// k_guide[z,g,:] = mean_{s<S} K[z,g,s,:]
__global__ __launch_bounds__(256) void kguide_kernel(PlanArgs a, Scratch sc) {
  __shared__ float red[16][kD];
  const int z = blockIdx.x / a.Hkv, g = blockIdx.x % a.Hkv;
  const int c = threadIdx.x & 15, r = threadIdx.x >> 4;
  const uint16_t* Kh = a.K + z * a.ks[0] + g * a.ks[1];
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int row = r; row < a.S; row += 16) {
    const u32x4 v = *reinterpret_cast<const u32x4*>(Kh + (int64_t)row * a.ks[2] + 8 * c);
#pragma unroll
    for (int q = 0; q < 4; ++q) { acc[2 * q] += bf16_lo(v[q]); acc[2 * q + 1] += bf16_hi(v[q]); }
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) red[r][8 * c + j] = acc[j];
  __syncthreads();
  if (threadIdx.x < kD) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += red[i][threadIdx.x];
    s *= 1.0f / (float)a.S;
    sc.kguide[(int64_t)blockIdx.x * kD + threadIdx.x] = s;
    if (a.k_guide) a.k_guide[(int64_t)blockIdx.x * kD + threadIdx.x] = s;
  }
}

// In-LDS bitonic sort of n2 (power of two) 64-bit keys, ascending.
__device__ inline void bitonic_sort_lds(uint64_t* keys, int n2, int tid, int nthreads) {
  for (int k = 2; k <= n2; k <<= 1) {
    for (int jj = k >> 1; jj > 0; jj >>= 1) {
      for (int t = tid; t < (n2 >> 1); t += nthreads) {
        const int i = ((t & ~(jj - 1)) << 1) | (t & (jj - 1));
        const int l = i | jj;
        const uint64_t x = keys[i], y = keys[l];
        const bool up = (i & k) == 0;
        if ((x > y) == up) { keys[i] = y; keys[l] = x; }
      }
      __syncthreads();
    }
  }
}

__device__ inline int next_pow2(int v) { int p = 1; while (p < v) p <<= 1; return p; }

// One workgroup per (z, h, n): q_mean, s_Q and Q_perm of the segment in one pass over Q.
__global__ __launch_bounds__(256) void pool_sq_sort_kernel(PlanArgs a, Scratch sc) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int n2 = next_pow2(a.S);
  uint64_t* keys = reinterpret_cast<uint64_t*>(smem);               // [n2]
  float* red = reinterpret_cast<float*>(smem + (size_t)n2 * 8);     // [16][128]

  const int G = a.H / a.Hkv;
  const int64_t row_id = blockIdx.x;                                // (z*H + h)*N + n
  const int n = (int)(row_id % a.N);
  const int h = (int)((row_id / a.N) % a.H);
  const int z = (int)(row_id / ((int64_t)a.N * a.H));
  const int g = h / G;
  const int tid = threadIdx.x, c = tid & 15, r = tid >> 4;
  const uint16_t* Qs = a.Q + z * a.qs[0] + h * a.qs[1] + (int64_t)n * a.S * a.qs[2];
  const float* kg = sc.kguide + ((int64_t)z * a.Hkv + g) * kD + 8 * c;
  float kgv[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) kgv[j] = kg[j];

  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int row = r; row < a.S; row += 16) {
    const u32x4 v = *reinterpret_cast<const u32x4*>(Qs + (int64_t)row * a.qs[2] + 8 * c);
    float dot = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float x0 = bf16_lo(v[q]), x1 = bf16_hi(v[q]);
      acc[2 * q] += x0; acc[2 * q + 1] += x1;
      dot = fmaf(x0, kgv[2 * q], dot);
      dot = fmaf(x1, kgv[2 * q + 1], dot);
    }
    dot += __shfl_xor(dot, 8);
    dot += __shfl_xor(dot, 4);
    dot += __shfl_xor(dot, 2);
    dot += __shfl_xor(dot, 1);
    if (c == 0) {
      keys[row] = sort_key(dot, (uint32_t)row);
      if (a.s_q) a.s_q[row_id * a.S + row] = dot;
    }
  }
  for (int i = a.S + tid; i < n2; i += 256) keys[i] = ~0ull;
  // ---- q_mean
#pragma unroll
  for (int j = 0; j < 8; ++j) red[r * kD + 8 * c + j] = acc[j];
  __syncthreads();
  if (tid < kD) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += red[i * kD + tid];
    s *= 1.0f / (float)a.S;
    sc.qmean[row_id * kD + tid] = s;
    if (a.q_mean) a.q_mean[row_id * kD + tid] = s;
    // exact three-way bf16 split (truncation keeps every step exact in fp32)
    const uint32_t u = __float_as_uint(s);
    const float hi = __uint_as_float(u & 0xffff0000u);
    const float r1 = s - hi;
    const float mid = __uint_as_float(__float_as_uint(r1) & 0xffff0000u);
    const float lo = r1 - mid;
    uint16_t* qs = sc.qsplit + row_id * 3 * kD;
    qs[tid] = (uint16_t)(__float_as_uint(hi) >> 16);
    qs[kD + tid] = (uint16_t)(__float_as_uint(mid) >> 16);
    qs[2 * kD + tid] = (uint16_t)(__float_as_uint(lo) >> 16);   // 8 bits left: exact
  }
  bitonic_sort_lds(keys, n2, tid, 256);
  for (int i = tid; i < a.S; i += 256) a.q_perm[row_id * a.S + i] = (int32_t)(uint32_t)keys[i];
}

// ---------------------------------------------------------------------------------------
// s_K scoring.  Workgroup = (z, g, row block of 32 rows, chunk of kTokChunk tokens); each of
// the 4 wavefronts takes 32-token column blocks of the chunk.  Row r of KV head g is
// (hq = r / N, n = r % N) and needs tokens t < n*S.
//   A (32 rows x 16 dims)  : q_mean split terms, lane (row = l%32, hh = l/32) holds dims
//                            64*hh + 8*kk .. +8 for contraction step kk
//   B (16 dims x 32 tokens): lane (token = l%32, hh) holds the same dims of its K row, i.e.
//                            each lane streams one contiguous 128-byte half row
//   C (32 rows x 32 tokens): register i of lane l = [row 8*(i/4) + 4*hh + i%4][token l%32]
template <int MODE>
__global__ __launch_bounds__(256) void score_kernel(PlanArgs a, Scratch sc) {
  const int G = a.H / a.Hkv;
  const int R = G * a.N;
  const int RB = (R + 31) / 32;
  const int nchunks = (a.L + kTokChunk - 1) / kTokChunk;
  int b = blockIdx.x;
  const int chunk = b % nchunks; b /= nchunks;
  const int rb = b % RB; b /= RB;
  const int g = b % a.Hkv;
  const int z = b / a.Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m_ = lane & 31, hh = lane >> 5;

  // token limit of the block's rows
  int limmax = 0;
  for (int i = 0; i < 32; ++i) {
    const int r = rb * 32 + i;
    if (r < R) limmax = max(limmax, (r % a.N) * a.S);
  }
  const int t_begin = chunk * kTokChunk;
  if (t_begin >= limmax) return;
  const int t_end = min(t_begin + kTokChunk, limmax);

  // per-register row data: rows of this lane's 16 accumulator registers
  int64_t row_id[16];      // (z*H + h)*N + n, or -1
  int lim[16];
  int64_t base[16];        // packed offset of the row inside s_k / pairs
  const int64_t P = kv_row_offset(a.N, a.S);
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int r = rb * 32 + 8 * (i >> 2) + 4 * hh + (i & 3);
    if (r < R) {
      const int hq = r / a.N, n = r % a.N;
      const int64_t zh = (int64_t)z * a.H + g * G + hq;
      row_id[i] = zh * a.N + n;
      lim[i] = n * a.S;
      base[i] = zh * P + kv_row_offset(n, a.S);
    } else {
      row_id[i] = -1; lim[i] = 0; base[i] = 0;
    }
  }
  float rhi[16], rscale[16];
  int rnb[16];
  if (MODE != 0) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      rhi[i] = 0.f; rscale[i] = 0.f; rnb[i] = 1;
      if (lim[i] > 0) {
        const float lo = ordered_to_float(sc.rowmin[row_id[i]]);
        rhi[i] = ordered_to_float(sc.rowmax[row_id[i]]);
        rnb[i] = row_buckets(lim[i] / a.S, a.S);
        const float range = rhi[i] - lo;
        rscale[i] = range > 0.f ? (float)rnb[i] / range : 0.f;
      }
    }
  }

  // A fragments: 3 split terms x 8 contraction steps
  bf16x8 af[3][8];
  {
    const int r = min(rb * 32 + m_, R - 1);
    const int hq = r / a.N, n = r % a.N;
    const int64_t rid = ((int64_t)z * a.H + g * G + hq) * a.N + n;
    const uint16_t* qs = sc.qsplit + rid * 3 * kD;
#pragma unroll
    for (int t = 0; t < 3; ++t)
#pragma unroll
      for (int kk = 0; kk < 8; ++kk)
        af[t][kk] = *reinterpret_cast<const bf16x8*>(qs + t * kD + 64 * hh + 8 * kk);
  }

  const uint16_t* Kh = a.K + z * a.ks[0] + g * a.ks[1];
  float vmin[16], vmax[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) { vmin[i] = INFINITY; vmax[i] = -INFINITY; }

  for (int t0 = t_begin + wave * 32; t0 < t_end; t0 += 4 * 32) {
    const int t = t0 + m_;                       // this lane's token (column)
    const uint16_t* krow = Kh + (int64_t)min(t, a.L - 1) * a.ks[2] + 64 * hh;
    bf16x8 kf[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) kf[kk] = *reinterpret_cast<const bf16x8*>(krow + 8 * kk);
    f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    // smallest term first so that the large products meet an accumulator that already
    // holds the corrections
#pragma unroll
    for (int tt = 2; tt >= 0; --tt)
#pragma unroll
      for (int kk = 0; kk < 8; ++kk)
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[tt][kk], kf[kk], acc, 0, 0, 0);

#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if (t < lim[i]) {
        const float s = acc[i];
        if (MODE == 0) {
          vmin[i] = fminf(vmin[i], s);
          vmax[i] = fmaxf(vmax[i], s);
          if (a.s_k) a.s_k[base[i] + t] = s;
        } else {
          int bk = (int)((rhi[i] - s) * rscale[i]);
          bk = min(max(bk, 0), rnb[i] - 1);
          if (MODE == 1) {
            atomicAdd(&sc.hist[row_id[i] * kNBMax + bk], 1u);
          } else {
            const uint32_t pos = atomicAdd(&sc.cursor[row_id[i] * kNBMax + bk], 1u);
            if (pos < (uint32_t)lim[i]) sc.pairs[base[i] + pos] = sort_key(s, (uint32_t)t);
            else sc.counters[2] = 1u;
          }
        }
      }
    }
  }
  if (MODE == 0) {
    // reduce over the 32 token lanes of each half, then one atomic per row
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      float lo = vmin[i], hi = vmax[i];
#pragma unroll
      for (int o = 16; o > 0; o >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, o));
        hi = fmaxf(hi, __shfl_xor(hi, o));
      }
      if (m_ == 0 && lim[i] > 0 && lo <= hi) {
        atomicMin(&sc.rowmin[row_id[i]], ordered_u32(lo));
        atomicMax(&sc.rowmax[row_id[i]], ordered_u32(hi));
      }
    }
  }
}

// Per prefix row: exclusive scan of the bucket histogram -> scatter cursors, and the list
// of spans handed to the sort kernels.
__global__ __launch_bounds__(64) void scan_kernel(PlanArgs a, Scratch sc) {
  const int64_t row_id = blockIdx.x;
  const int n = (int)(row_id % a.N);
  if (n == 0) return;
  if (threadIdx.x != 0) return;
  const int nb = row_buckets(n, a.S);
  uint32_t* hist = sc.hist + row_id * kNBMax;
  uint32_t* cur = sc.cursor + row_id * kNBMax;
  uint32_t off = 0, span_begin = 0;
  for (int b = 0; b < nb; ++b) {
    const uint32_t cnt = hist[b];
    cur[b] = off;
    if (cnt > (uint32_t)kSpanCap) {
      if (off > span_begin) {
        const uint32_t s = atomicAdd(&sc.counters[0], 1u);
        if ((int64_t)s < sc.max_spans) sc.spans[s] = make_int4((int)row_id, (int)span_begin, (int)off, 0);
      }
      const uint32_t s = atomicAdd(&sc.counters[1], 1u);
      if ((int64_t)s < sc.max_spans) sc.bigspans[s] = make_int4((int)row_id, (int)off, (int)(off + cnt), 0);
      span_begin = off + cnt;
    } else if (off + cnt - span_begin > (uint32_t)kSpanCap) {
      const uint32_t s = atomicAdd(&sc.counters[0], 1u);
      if ((int64_t)s < sc.max_spans) sc.spans[s] = make_int4((int)row_id, (int)span_begin, (int)off, 0);
      span_begin = off;
    }
    off += cnt;
  }
  if (off > span_begin) {
    const uint32_t s = atomicAdd(&sc.counters[0], 1u);
    if ((int64_t)s < sc.max_spans) sc.spans[s] = make_int4((int)row_id, (int)span_begin, (int)off, 0);
  }
}

__device__ inline int64_t row_base(const PlanArgs& a, int64_t row_id) {
  const int n = (int)(row_id % a.N);
  const int64_t zh = row_id / a.N;
  return zh * kv_row_offset(a.N, a.S) + kv_row_offset(n, a.S);
}

__global__ __launch_bounds__(256) void span_sort_kernel(PlanArgs a, Scratch sc) {
  __shared__ uint64_t keys[kSpanCap];
  if (blockIdx.x >= sc.counters[0]) return;
  const int4 sp = sc.spans[blockIdx.x];
  const int64_t base = row_base(a, sp.x) + sp.y;
  const int len = sp.z - sp.y;
  const int n2 = next_pow2(len);
  for (int i = threadIdx.x; i < n2; i += 256) keys[i] = i < len ? sc.pairs[base + i] : ~0ull;
  __syncthreads();
  bitonic_sort_lds(keys, n2, threadIdx.x, 256);
  for (int i = threadIdx.x; i < len; i += 256) a.kv_perm[base + i] = (int32_t)(uint32_t)keys[i];
}

// Fallback: stable LSD radix sort (8 passes of 8 bits) of one oversized bucket by one
// workgroup, ping-ponging between the pair scratch and a private buffer.
__global__ __launch_bounds__(256) void big_sort_kernel(PlanArgs a, Scratch sc) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t basep[256];
  __shared__ uint32_t dig[256];
  const int tid = threadIdx.x;
  const uint32_t nbig = min(sc.counters[1], (uint32_t)sc.max_spans);
  uint64_t* mine = sc.alt + (int64_t)blockIdx.x * a.L;
  for (uint32_t w = blockIdx.x; w < nbig; w += gridDim.x) {
    const int4 sp = sc.bigspans[w];
    const int64_t base = row_base(a, sp.x) + sp.y;
    const int len = sp.z - sp.y;
    uint64_t* src = sc.pairs + base;
    uint64_t* dst = mine;
    for (int pass = 0; pass < 8; ++pass) {
      const int shift = 8 * pass;
      hist[tid] = 0;
      __syncthreads();
      for (int i = tid; i < len; i += 256) atomicAdd(&hist[(src[i] >> shift) & 255u], 1u);
      __syncthreads();
      if (tid == 0) {
        uint32_t o = 0;
        for (int d = 0; d < 256; ++d) { basep[d] = o; o += hist[d]; }
      }
      __syncthreads();
      for (int c0 = 0; c0 < len; c0 += 256) {
        const int i = c0 + tid;
        uint64_t key = 0;
        uint32_t d = 256u;
        if (i < len) { key = src[i]; d = (uint32_t)(key >> shift) & 255u; }
        dig[tid] = d;
        __syncthreads();
        uint32_t pos = 0;
        if (i < len) {
          uint32_t rank = 0;
          for (int t = 0; t < tid; ++t) rank += (dig[t] == d) ? 1u : 0u;
          pos = basep[d] + rank;
        }
        __syncthreads();
        if (i < len) { dst[pos] = key; atomicMax(&basep[d], pos + 1); }
        __syncthreads();
      }
      uint64_t* t = src; src = dst; dst = t;
      __threadfence();
      __syncthreads();
    }
    // 8 passes: the sorted data is back in the pair scratch
    for (int i = tid; i < len; i += 256) a.kv_perm[base + i] = (int32_t)(uint32_t)sc.pairs[base + i];
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------
hipError_t launch_plan(const PlanArgs& a, hipStream_t stream) {
  const Scratch sc = carve(a.scratch, a.Z, a.H, a.Hkv, a.L, a.S);
  if (sc.total > a.scratch_bytes) return hipErrorInvalidValue;
  const int64_t rows = (int64_t)a.Z * a.H * a.N;
  const int G = a.H / a.Hkv;

  {
    const int64_t nthr = rows * kNBMax;
    hipLaunchKernelGGL(init_kernel, dim3((unsigned)((nthr + 255) / 256)), dim3(256), 0, stream, sc, rows);
  }
  hipLaunchKernelGGL(kguide_kernel, dim3(a.Z * a.Hkv), dim3(256), 0, stream, a, sc);
  {
    int n2 = 1;
    while (n2 < a.S) n2 <<= 1;
    const size_t lds = (size_t)n2 * 8 + 16 * kD * 4;
    static bool attr_set = false;
    if (!attr_set) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&pool_sq_sort_kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 8192 * 8 + 16 * kD * 4);
      if (e != hipSuccess) return e;
      attr_set = true;
    }
    hipLaunchKernelGGL(pool_sq_sort_kernel, dim3((unsigned)rows), dim3(256), lds, stream, a, sc);
  }
  if (a.N > 1) {
    const int RB = (G * a.N + 31) / 32;
    const int nchunks = (a.L + kTokChunk - 1) / kTokChunk;
    const dim3 grid((unsigned)((int64_t)a.Z * a.Hkv * RB * nchunks));
    hipLaunchKernelGGL(score_kernel<0>, grid, dim3(256), 0, stream, a, sc);
    hipLaunchKernelGGL(score_kernel<1>, grid, dim3(256), 0, stream, a, sc);
    hipLaunchKernelGGL(scan_kernel, dim3((unsigned)rows), dim3(64), 0, stream, a, sc);
    hipLaunchKernelGGL(score_kernel<2>, grid, dim3(256), 0, stream, a, sc);
    hipLaunchKernelGGL(span_sort_kernel, dim3((unsigned)sc.max_spans), dim3(256), 0, stream, a, sc);
    hipLaunchKernelGGL(big_sort_kernel, dim3(kBigGrid), dim3(256), 0, stream, a, sc);
  }
  return hipGetLastError();
}

}  // namespace s2o
