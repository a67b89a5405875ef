// S2O ranking stage for gfx950 (paper Sec. 3.1, Alg. 1, Eqs. (1)-(2)).
//
//   kguide_kernel        k_guide = mean of the first key segment (k_mean[0]).
//   pool_sq_sort_kernel  one workgroup per (z, h, segment): a single pass over the
//                        segment's Q rows gives q_mean and s_Q; the S scores are then
//                        Argsort-ed in LDS (bitonic network on 64-bit keys) -> Q_perm.
//   score_kernel         s_K[n, t] = <q_mean[n], K[t]> as an MFMA contraction per KV head:
//                        columns = (query head of the group, segment), rows = key tokens
//                        staged through LDS.  q_mean is split exactly into three bf16 terms
//                        so that bf16 MFMA reproduces the fp32 x bf16 products exactly (fp32
//                        accumulation).  The scores are stored (in the caller's s_K array or
//                        in scratch) together with one sampled score per 64 tokens.
//                        The Argsort of a prefix row (up to L - S scores) is a sample sort:
//                        buckets are delimited by splitters taken from a sorted sample of
//                        the row, so their populations are balanced for any distribution.
//   splitter_kernel      per prefix row: sorts the sample in LDS and keeps every
//                        (sample size / buckets)-th value as a splitter.
//   scatter_kernel       per (row, cell of up to 1024 tokens): (key, token) pairs to their
//                        bucket.  Every bucket of a row owns a region of twice the average
//                        population; the cell counts its buckets in LDS, claims a run in each
//                        region with one atomic add on the row's cursor, and writes its pairs
//                        staged in LDS sorted by bucket, so that the global stores are runs,
//                        not scatters.  No counting pass over the scores, no offset scan.
//   span_kernel          per prefix row: the final cursors are the bucket populations; cuts
//                        them into spans (runs of consecutive buckets that fit the LDS sort).
//   count_kernel, scan_exact_kernel, scatter_exact_kernel
//                        the exact path for rows in which a bucket outgrew its region (many
//                        equal scores): bucket counts per cell, run offsets (bucket-major,
//                        cell-minor), scatter to a compact layout.  They loop over a list of
//                        such rows, which is normally empty.
//   span_sort_kernel     sorts each span in LDS and writes the token indices at their
//                        final ranks -> KV_perm.  Linear-time: a second, fine bucketing on
//                        the score value leaves a few keys per sub-bucket, which are ranked by
//                        direct comparison; a span whose keys pile up in one sub-bucket
//                        (many equal scores) falls back to a bitonic network.
//   big_sort_kernel      fallback for a bucket that alone exceeds the LDS sort (e.g. all
//                        scores equal): a stable LSD radix sort by one workgroup.
//
// Argsort semantics: descending score, ties by ascending index, -0 == +0.  Every sort works
// on the 64-bit key (~ordered(score)) << 32 | index, whose ascending order is exactly
// that order, so no stability property is needed anywhere.
#include "s2o_internal.h"

namespace s2o {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kD = 128;
constexpr int kNBMax = 64;         // buckets per prefix row (upper bound)
constexpr int kBucketAvg = 2048;   // target average bucket population
constexpr int kSampleStride = 64;  // one sampled score per this many tokens
constexpr int kSpanCap = 4096;     // elements one span_sort workgroup sorts in LDS
constexpr int kSubBuckets = 2048;  // fine buckets of the in-LDS sort
constexpr int kSubMax = 64;        // a fuller sub-bucket sends the span to the bitonic fallback
constexpr int kChunkMax = 1024;    // key tokens per score workgroup (halved while the grid is too small)
constexpr int kCellMax = 1024;     // key tokens per (row, cell) of the scatter: four per thread (512 tokens and
                                   // 128 threads: 489 against 476 us at 128K)
constexpr int kScatterThreads = kCellMax / 4;
constexpr int kSub = 128;          // key tokens per LDS tile of the score kernel
constexpr int kScoreWaves = 4;     // wavefronts (row blocks of 32) of a score workgroup.  8 would let all 4 x 64 rows
                                   // of a KV head at 128K share one pass over its K rows (295 against 307 us alone),
                                   // but an 8-wavefront workgroup of 200 registers needs a whole CU at once and
                                   // starves beside the own-segment pass on the second stream (up to 3 ms)
constexpr int kKStride = 136;      // bf16 elements per K row in LDS (272 B)
constexpr int kBigGrid = 64;       // workgroups of the fallback sort
constexpr int kRedoGrid = 2048;    // workgroups of the exact path's kernels (they loop over the redo list)

__host__ __device__ inline int row_buckets(int64_t len) {
  const int64_t nb = len / kBucketAvg;
  return nb < 1 ? 1 : (nb > kNBMax ? kNBMax : (int)nb);
}

// Layout of the (key, token) pairs between the scatter and the sorts.  Every bucket of a row owns
// a region of bucket_cap(len) slots, twice the average population, and the workgroups of the
// scatter claim runs inside it from a cursor, so no counting pass over the scores is needed to
// find a run's place.  (The splitters are every 32nd value of a sorted 1-in-64 sample, so a
// bucket's population scatters like a Gamma(32) variable around the mean, sigma = 18 %: twice
// the mean is 5.7 sigma away; one and a half times would send one row in five to the exact
// path.)  A row in which some bucket does outgrow its region -- many equal scores -- is laid out
// again by the exact path (count, offsets, scatter), compactly, from the start of its regions.
// region_base(n): first slot of row n inside its head, a closed-form upper bound of the sum of
// the earlier rows' regions (nb * cap < 2 * len + 16 * nb; regions start on 128-byte
// boundaries).
__host__ __device__ inline uint32_t bucket_cap(int64_t len) {
  const int64_t avg = len / row_buckets(len);
  return (uint32_t)((2 * avg + 15) & ~(int64_t)15);
}
__host__ __device__ inline int64_t region_base(int64_t n, int64_t S, int64_t L, int nc) {
  return nc ? n * (2 * L + 16 * kNBMax) : 2 * kv_row_offset(n, S) + n * 16 * kNBMax;
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
  float* kguide;      // [Z*Hkv][kGuideParts][128] partial column sums of the first key segment
  float* qmean;       // [Z*H*N*128]
  uint16_t* qsplit;   // [Z*H*N][3][128] bf16
  float* samples;     // [Z*H*N][L/64] one score per 64 tokens of the row's prefix
  float* splitters;   // [Z*H*N][kNBMax] descending; entries past the row's buckets are -inf
  uint16_t* chist;    // [Z*H*N][maxch][kNBMax] bucket counts per cell of `cell` tokens
  uint32_t* coffs;    // same shape: offset of the cell inside its row
  uint32_t* counters; // [0]=#spans [1]=#big spans [2]=error flag [3]=#rows redone by the exact path
  uint32_t* cursor;   // [Z*H*N][kNBMax] pairs claimed so far in each bucket's region (= its population at the end)
  uint32_t* rowflag;  // [Z*H*N] != 0: a bucket of the row outgrew its region
  uint32_t* bst;      // [Z*H*N][kNBMax+1] rank at which each bucket of the row starts
  int32_t* redo;      // [Z*H*N] rows whose buckets are laid out again by the exact (counting) path
  int4* spans;        // [max_spans][2]  (row, first rank, end rank, w), (starts of the span's first four buckets)
  int4* bigspans;     // [max_spans]
  float* sk;          // [Z*H*P] s_K, used when the caller does not ask for the scores
  uint64_t* pairs;    // [Z*H][region_base(N)]: per row one region per bucket (see bucket_cap)
  int64_t pairs_per_head;
  uint64_t* alt;      // [kBigGrid * L]
  int64_t max_spans;
  int maxch;          // cells per row
  int cell;           // key tokens per (row, cell) of the bucket counts
  int chunk;          // key tokens per score workgroup: kChunkMax, less for short sequences
  size_t total;
};

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static Scratch carve(void* base, int Z, int H, int Hkv, int L, int S, int non_causal) {
  const int64_t N = L / S;
  const int64_t rows = (int64_t)Z * H * N;
  const int64_t P = kv_rows_total(N, S, L, non_causal);
  Scratch s;
  s.max_spans = (int64_t)Z * H * (3 * P / kSpanCap + 2 * N) + 8;
  // one workgroup per (KV head, 128 rows, chunk): keep at least ~1024 of them in the grid
  {
    const int64_t rbg = ((int64_t)(H / Hkv) * N + 32 * kScoreWaves - 1) / (32 * kScoreWaves);
    s.chunk = kChunkMax;
    while (s.chunk > kSub && (int64_t)Z * Hkv * rbg * ((L + s.chunk - 1) / s.chunk) < 1024) s.chunk /= 2;
  }
  // bucket counts are kept per (row, cell of tokens); one workgroup of the counting and scatter
  // passes handles one cell: as large as the staging area allows unless the grid gets too small
  s.cell = kCellMax;
  while (s.cell > 256 && rows * (((non_causal ? L : L / 2) + s.cell - 1) / s.cell) < 2048) s.cell /= 2;
  s.maxch = (L + s.cell - 1) / s.cell;
  size_t off = 0;
  // (integer arithmetic: the size query carves from a null base)
  auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return (char*)((uintptr_t)base + o); };
  s.kguide = (float*)take((size_t)Z * Hkv * 8 * kD * 4);
  s.qmean = (float*)take((size_t)rows * kD * 4);
  s.qsplit = (uint16_t*)take((size_t)rows * 3 * kD * 2);
  s.samples = (float*)take((size_t)rows * (L / kSampleStride) * 4);
  s.splitters = (float*)take((size_t)rows * kNBMax * 4);
  s.chist = (uint16_t*)take((size_t)rows * s.maxch * kNBMax * 2);
  s.coffs = (uint32_t*)take((size_t)rows * s.maxch * kNBMax * 4);
  s.counters = (uint32_t*)take(64);
  s.cursor = (uint32_t*)take((size_t)rows * kNBMax * 4);
  s.rowflag = (uint32_t*)take((size_t)rows * 4);
  s.bst = (uint32_t*)take((size_t)rows * (kNBMax + 1) * 4);
  s.redo = (int32_t*)take((size_t)rows * 4);
  s.spans = (int4*)take((size_t)s.max_spans * 32);
  s.bigspans = (int4*)take((size_t)s.max_spans * 16);
  s.sk = (float*)take((size_t)Z * H * P * 4);
  s.pairs_per_head = region_base(N, S, L, non_causal);
  s.pairs = (uint64_t*)take((size_t)Z * H * s.pairs_per_head * 8);
  s.alt = (uint64_t*)take((size_t)kBigGrid * L * 8);
  s.total = off;
  return s;
}

size_t plan_scratch_bytes(int Z, int H, int Hkv, int L, int S, int non_causal) {
  return carve(nullptr, Z, H, Hkv, L, S, non_causal).total;
}

// ---------------------------------------------------------------------------------------
// Built-in scratch for callers that cannot allocate (s2o_plan_static): one array per GPU, held
// from the moment the library is loaded there until the process ends.  The name below is a
// host-side stand-in, not a device address: host code only ever uses the address that
// hipGetSymbolAddress reports for the current device.
static __device__ __align__(256) unsigned char scratch[kStaticPlanScratchBytes];

hipError_t static_plan_scratch(void** ptr) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* addr[kMaxDevices] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!addr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    addr[dev] = p;
  }
  *ptr = addr[dev];
  return hipSuccess;
}

// ---------------------------------------------------------------------------------------
__global__ void init_kernel(Scratch s, int64_t rows, int32_t* status) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < 16) s.counters[i] = 0;
  if (i == 0 && status) *status = 0;
}

// A broken invariant (see the S2O_PLAN_* bits) is recorded in the scratch counters and, if the
// caller gave one, in the status word; nothing is ever dropped silently.
__device__ inline void raise(const PlanArgs& a, const Scratch& sc, uint32_t bit) {
  atomicOr(&sc.counters[2], bit);
  if (a.status) atomicOr(reinterpret_cast<unsigned int*>(a.status), bit);
}

// k_guide[z,g,:] = mean_{s<S} K[z,g,s,:]
constexpr int kGuideParts = 8;     // workgroups per KV head summing the first key segment

// Partial column sums of the first key segment: workgroup (z, g, part) adds the rows of its
// eighth of the segment; the consumers add the eight partial sums in a fixed order, so k_guide
// is reproducible bit for bit without a serial pass over the segment by one workgroup.
__global__ __launch_bounds__(256) void kguide_kernel(PlanArgs a, Scratch sc) {
  __shared__ float red[16][kD];
  const int unit = blockIdx.x / kGuideParts, part = blockIdx.x % kGuideParts;
  const int z = unit / a.Hkv, g = unit % a.Hkv;
  const int c = threadIdx.x & 15, r = threadIdx.x >> 4;
  const uint16_t* Kh = a.K + z * a.ks[0] + g * a.ks[1];
  const int rows = a.S / kGuideParts;            // S is a multiple of 64
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int row = part * rows + r; row < (part + 1) * rows; row += 16) {
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
    sc.kguide[(int64_t)blockIdx.x * kD + threadIdx.x] = s;
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
  float* red = reinterpret_cast<float*>(smem + (size_t)n2 * 8);     // [4 wavefronts][128]

  const int G = a.H / a.Hkv;
  const int64_t row_id = blockIdx.x;                                // (z*H + h)*N + n
  const int n = (int)(row_id % a.N);
  const int h = (int)((row_id / a.N) % a.H);
  const int z = (int)(row_id / ((int64_t)a.N * a.H));
  const int g = h / G;
  const int tid = threadIdx.x, c = tid & 15, r = tid >> 4;
  const uint16_t* Qs = a.Q + z * a.qs[0] + h * a.qs[1] + (int64_t)n * a.S * a.qs[2];
  // k_guide = mean of the first key segment, from the partial sums in a fixed order
  const float* kg = sc.kguide + ((int64_t)z * a.Hkv + g) * kGuideParts * kD + 8 * c;
  float kgv[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    float t = 0.f;
#pragma unroll
    for (int pp = 0; pp < kGuideParts; ++pp) t += kg[pp * kD + j];
    kgv[j] = t * (1.0f / (float)a.S);
  }
  if (a.k_guide && n == 0 && h % G == 0 && r == 0) {
#pragma unroll
    for (int j = 0; j < 8; ++j) a.k_guide[((int64_t)z * a.Hkv + g) * kD + 8 * c + j] = kgv[j];
  }

  // the scatter's bucket cursors of this row start at zero
  if (tid < kNBMax) sc.cursor[row_id * kNBMax + tid] = 0u;
  if (tid == kNBMax) sc.rowflag[row_id] = 0u;

  // Four rows of a thread per trip, all four 16-byte loads issued before the first is used
  // (S is a multiple of 64: no tail).
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int row0 = r; row0 < a.S; row0 += 64) {
    u32x4 v4[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      v4[u] = *reinterpret_cast<const u32x4*>(Qs + (int64_t)(row0 + 16 * u) * a.qs[2] + 8 * c);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int row = row0 + 16 * u;
      const u32x4 v = v4[u];
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
  }
  for (int i = a.S + tid; i < n2; i += 256) keys[i] = ~0ull;
  // ---- q_mean: column sums over the wavefront's four row groups, then over the wavefronts
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    acc[j] += __shfl_xor(acc[j], 16);
    acc[j] += __shfl_xor(acc[j], 32);
  }
  if ((tid & 63) < 16) {
#pragma unroll
    for (int j = 0; j < 8; ++j) red[(tid >> 6) * kD + 8 * c + j] = acc[j];
  }
  __syncthreads();
  if (tid < kD) {
    float s = (red[tid] + red[kD + tid]) + (red[2 * kD + tid] + red[3 * kD + tid]);
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
// s_K scoring.  Workgroup = (z, g, group of kScoreWaves row blocks, chunk of sc.chunk tokens);
// wavefront w owns row block kScoreWaves*group + w (32 rows of the contraction's N side) and keeps
// its q_mean split fragments in registers for the whole chunk; the chunk's K rows pass through
// LDS in tiles of kSub tokens shared by the wavefronts.  Row r of KV head g is (hq = r / N,
// n = r % N) and needs tokens t < n*S.
//   A (32 tokens x 16 dims): K tile rows from LDS, lane (token = l%32, hh = l/32) reads dims
//                            16*kk + 8*hh .. +8
//   B (16 dims x 32 rows)  : q_mean split terms, lane (row = l%32, hh) holds the same dims
//   C (32 tokens x 32 rows): register i of lane l = [token 8*(i/4) + 4*hh + i%4][row l%32],
//                            so a lane sees one row only and its meta data are scalars
__global__ __launch_bounds__(64 * kScoreWaves) void score_kernel(PlanArgs a, Scratch sc) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* Kt = reinterpret_cast<uint16_t*>(smem);                          // [kSub][kKStride]

  const int G = a.H / a.Hkv;
  const int R = G * a.N;
  const int nchunks = (a.L + sc.chunk - 1) / sc.chunk;
  // all work on one KV head goes to one XCD (block ids are dealt round-robin to the 8 XCDs):
  // the row blocks of a head read the same K chunks
  int unit, rest;
  {
    const int U = a.Z * a.Hkv, b = blockIdx.x;
    if (U % 8 == 0) {
      const int xcd = b & 7, idx = b >> 3, per = U / 8;
      unit = (idx % per) * 8 + xcd;
      rest = idx / per;
    } else {
      unit = b % U;
      rest = b / U;
    }
  }
  const int chunk = rest % nchunks;
  const int rbg = rest / nchunks;
  const int g = unit % a.Hkv, z = unit / a.Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m_ = lane & 31, hh = lane >> 5;
  const int rb = kScoreWaves * rbg + wave;

  auto row_limit = [&](int r) { return r < R ? (int)kv_row_len(r % a.N, a.S, a.L, a.non_causal) : 0; };
  // token limits: of the workgroup's rows (uniform) and of this wavefront's rows
  int lim_wg = 0, lim_wave = 0;
  for (int i = 0; i < 32 * kScoreWaves; ++i) lim_wg = max(lim_wg, row_limit(32 * kScoreWaves * rbg + i));
  for (int i = 0; i < 32; ++i) lim_wave = max(lim_wave, row_limit(32 * rb + i));
  const int t_begin = chunk * sc.chunk;
  if (t_begin >= lim_wg) return;
  const int t_end = min(t_begin + sc.chunk, lim_wg);

  // this lane's row
  const int r = 32 * rb + m_;
  const int lim = row_limit(r);
  const int rr = min(r, R - 1);
  const int64_t zh = (int64_t)z * a.H + g * G + rr / a.N;
  const int64_t row_id = zh * a.N + rr % a.N;
  const int64_t base = zh * kv_rows_total(a.N, a.S, a.L, a.non_causal) +
                       kv_row_start(rr % a.N, a.S, a.L, a.non_causal);
  float* skdst = (a.s_k ? a.s_k : sc.sk) + base;

  // B fragments: 3 split terms x 8 contraction steps
  bf16x8 bq[3][8];
  {
    const uint16_t* qs = sc.qsplit + row_id * 3 * kD;
#pragma unroll
    for (int t = 0; t < 3; ++t)
#pragma unroll
      for (int kk = 0; kk < 8; ++kk)
        bq[t][kk] = *reinterpret_cast<const bf16x8*>(qs + t * kD + 16 * kk + 8 * hh);
  }
  const int samples_per_row = a.L / kSampleStride;

  // K tile loader: thread (c, q) moves 16-byte chunk c of rows q, q+16, ...
  const uint16_t* Kh = a.K + z * a.ks[0] + g * a.ks[1];
  const int c = tid & 15, q = tid >> 4;
  constexpr int kLoadRows = 4 * kScoreWaves;      // tile rows one pass of the loader covers
  u32x4 kreg[kSub / kLoadRows];
  auto load_tile = [&](int t0) {
#pragma unroll
    for (int s = 0; s < kSub / kLoadRows; ++s) {
      const int t = min(t0 + q + kLoadRows * s, a.L - 1);
      kreg[s] = *reinterpret_cast<const u32x4*>(Kh + (int64_t)t * a.ks[2] + 8 * c);
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int s = 0; s < kSub / kLoadRows; ++s)
      *reinterpret_cast<u32x4*>(Kt + (q + kLoadRows * s) * kKStride + 8 * c) = kreg[s];
  };

  load_tile(t_begin);
  for (int t0 = t_begin; t0 < t_end; t0 += kSub) {
    __syncthreads();                       // previous tile fully consumed
    store_tile();
    __syncthreads();
    if (t0 + kSub < t_end) load_tile(t0 + kSub);
    if (t0 < lim_wave) {
#pragma unroll 1
      for (int sb = 0; sb < kSub / 32; ++sb) {
        f32x16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
        bf16x8 ka[8];
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
          ka[kk] = *reinterpret_cast<const bf16x8*>(Kt + (32 * sb + m_) * kKStride + 16 * kk + 8 * hh);
        // smallest term first so that the large products meet an accumulator that already
        // holds the corrections
#pragma unroll
        for (int tt = 2; tt >= 0; --tt)
#pragma unroll
          for (int kk = 0; kk < 8; ++kk)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kk], bq[tt][kk], acc, 0, 0, 0);
        // lim is a multiple of 64, so a 32-token block is valid for this row as a whole or not at all
        if (t0 + 32 * sb < lim) {
          // sample: one token of every 64, at a position that varies from block to block
          const int blk = (t0 + 32 * sb) / kSampleStride;
          const int off = ((blk * 37 + 11) & 63) - 32 * (sb & 1);   // offset inside this 32-token block
          if (off >= 0 && off < 32 && ((off >> 2) & 1) == hh) {
            const int idx = 4 * (off >> 3) + (off & 3);               // register holding that token
            float v = acc[0];
#pragma unroll
            for (int i = 1; i < 16; ++i) v = idx == i ? acc[i] : v;
            sc.samples[row_id * samples_per_row + blk] = v;
          }
          // the four registers of a group are four consecutive tokens
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            const int t = t0 + 32 * sb + 8 * i4 + 4 * hh;
            const f32x4 v = {acc[4 * i4], acc[4 * i4 + 1], acc[4 * i4 + 2], acc[4 * i4 + 3]};
            *reinterpret_cast<f32x4*>(skdst + t) = v;
          }
        }
      }
    }
  }
}

__device__ inline int64_t row_base(const PlanArgs& a, int64_t row_id) {
  const int n = (int)(row_id % a.N);
  const int64_t zh = row_id / a.N;
  return zh * kv_rows_total(a.N, a.S, a.L, a.non_causal) + kv_row_start(n, a.S, a.L, a.non_causal);
}

// First pair slot of a row's regions.
__device__ inline uint64_t* row_pairs(const PlanArgs& a, const Scratch& sc, int64_t row_id) {
  const int n = (int)(row_id % a.N);
  return sc.pairs + (row_id / a.N) * sc.pairs_per_head + region_base(n, a.S, a.L, a.non_causal);
}
// The same two for a row given as (head index zh = z*H + h, segment n): the sorts look rows up
// once per span and per thread, where the 64-bit divisions above would cost as much as ranking
// a few keys.
__device__ inline int64_t row_base(const PlanArgs& a, int zh, int n) {
  return (int64_t)zh * kv_rows_total(a.N, a.S, a.L, a.non_causal) + kv_row_start(n, a.S, a.L, a.non_causal);
}
__device__ inline uint64_t* row_pairs(const PlanArgs& a, const Scratch& sc, int zh, int n) {
  return sc.pairs + (int64_t)zh * sc.pairs_per_head + region_base(n, a.S, a.L, a.non_causal);
}

// Bucket of a score = number of the row's (descending) splitters above it.  Two levels, both
// by counting instead of a dependent binary search: every 8th splitter sits in a register
// (top[k] = splitter 8k+7), the group of 7 below the hit comes from LDS with two 16-byte reads.
__device__ inline int bucket_of_score(const float* spl, const float (&top)[7], float sv) {
  int gi = 0;
#pragma unroll
  for (int k = 0; k < 7; ++k) gi += top[k] > sv ? 1 : 0;
  const f32x4 lo = *reinterpret_cast<const f32x4*>(spl + 8 * gi);
  const f32x4 hi = *reinterpret_cast<const f32x4*>(spl + 8 * gi + 4);
  int bk = 8 * gi;
  bk += lo[0] > sv ? 1 : 0; bk += lo[1] > sv ? 1 : 0; bk += lo[2] > sv ? 1 : 0; bk += lo[3] > sv ? 1 : 0;
  bk += hi[0] > sv ? 1 : 0; bk += hi[1] > sv ? 1 : 0; bk += hi[2] > sv ? 1 : 0;
  return bk;
}

// Counting and scatter passes of the sample sort, streaming over the stored scores: one
// workgroup per (prefix row, cell of sc.cell tokens), threads striding over the tokens.  All
// lanes work on the same row, so the splitter reads are broadcasts, the kernels need a few
// dozen registers, and enough wavefronts are resident to hide the LDS round trips
// (re-computing the scores with MFMA in these passes kept them latency-bound at a quarter
// of the issue rate).
// Exact path, pass 1 (only for the rows on the redo list): bucket counts per cell.
__global__ __launch_bounds__(256) void count_kernel(PlanArgs a, Scratch sc, int64_t rows) {
  __shared__ __attribute__((aligned(16))) float spl[kNBMax];
  __shared__ uint32_t cnt[kNBMax];
  const int64_t nredo = min((int64_t)sc.counters[3], rows);
  for (int64_t item = blockIdx.x; item < nredo * sc.maxch; item += gridDim.x) {
    const int64_t row_id = sc.redo[item / sc.maxch];
    const int cellno = (int)(item % sc.maxch);
    const int lim = (int)kv_row_len(row_id % a.N, a.S, a.L, a.non_causal);   // keys this row ranks
    const int t_begin = cellno * sc.cell;
    if (t_begin >= lim) continue;
    const int t_end = min(t_begin + sc.cell, lim);
    const int tid = threadIdx.x;
    // four consecutive scores per thread, requested before the splitters are staged (cells and
    // prefix lengths are multiples of 4 tokens and rows start 16-byte aligned)
    const float* sk = (a.s_k ? a.s_k : sc.sk) + row_base(a, row_id);
    const int t0 = t_begin + 4 * tid;
    f32x4 sv4 = {0.f, 0.f, 0.f, 0.f};
    if (t0 < t_end) sv4 = *reinterpret_cast<const f32x4*>(sk + t0);
    __syncthreads();                      // the previous item's counters have been written out
    if (tid < kNBMax) {
      spl[tid] = sc.splitters[row_id * kNBMax + tid];
      cnt[tid] = 0u;
    }
    __syncthreads();
    float top[7];
#pragma unroll
    for (int k = 0; k < 7; ++k) top[k] = spl[8 * k + 7];
    if (t0 < t_end) {
#pragma unroll
      for (int e = 0; e < 4; ++e) atomicAdd(&cnt[bucket_of_score(spl, top, sv4[e])], 1u);
    }
    __syncthreads();
    if (tid < kNBMax) sc.chist[(row_id * sc.maxch + cellno) * kNBMax + tid] = (uint16_t)cnt[tid];
  }
}

// Scatter: the cell's (key, token) pairs are first placed in LDS sorted by bucket (rank from an
// LDS cursor that starts at the bucket's offset inside the cell), each with its destination;
// the staged pairs are then written out in staged order, so that the lanes of a store
// instruction hit runs of consecutive addresses (a bucket's run of this cell) instead of 64
// different cache lines.
//
// scatter_kernel (every row): the cell counts its own buckets in LDS, claims a run for each in
// the bucket's region with one atomic add on the row's cursor and writes there.  The order of
// the runs inside a region depends on which workgroup claims first; the sorts that follow order
// by (score, token), so the maps do not.  A bucket that would outgrow its region marks the row
// for the exact path and writes nothing.
constexpr int kCellsPerWg = 1;     // consecutive cells of a row per scatter workgroup (a later cell's scores are
                                   // requested before the earlier cell is worked on).  2 is slower at 128K (532
                                   // against 476 us): the kernel lives on the number of independent workgroups
                                   // in flight, not on the latency of one

__global__ __launch_bounds__(kScatterThreads) void scatter_kernel(PlanArgs a, Scratch sc) {
  __shared__ __attribute__((aligned(16))) float spl[kNBMax];
  __shared__ uint32_t cnt[kNBMax];              // population of each bucket in this cell
  __shared__ uint32_t cur[kNBMax];              // first staging slot of each bucket
  __shared__ uint32_t delta[kNBMax];            // slot in the row's regions - staging slot; ~0: no room
  __shared__ uint64_t stage[kCellMax];
  __shared__ uint32_t sdst[kCellMax];
  const int cgroups = (sc.maxch + kCellsPerWg - 1) / kCellsPerWg;
  const int64_t row_id = blockIdx.x / cgroups;
  const int cell0 = (int)(blockIdx.x % cgroups) * kCellsPerWg;
  const int lim = (int)kv_row_len(row_id % a.N, a.S, a.L, a.non_causal);
  if (cell0 * sc.cell >= lim) return;
  const int tid = threadIdx.x;
  const float* sk = (a.s_k ? a.s_k : sc.sk) + row_base(a, row_id);
  // four consecutive scores per thread (cells and prefix lengths are multiples of 4 tokens and
  // rows start 16-byte aligned)
  auto load4 = [&](int cellno) {
    const int t = cellno * sc.cell + 4 * tid;
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (t < min((cellno + 1) * sc.cell, lim)) v = *reinterpret_cast<const f32x4*>(sk + t);
    return v;
  };
  f32x4 sv4 = load4(cell0);
  if (tid < kNBMax) {
    spl[tid] = sc.splitters[row_id * kNBMax + tid];
    cnt[tid] = 0u;
  }
  __syncthreads();
  float top[7];
#pragma unroll
  for (int k = 0; k < 7; ++k) top[k] = spl[8 * k + 7];
  const uint32_t cap = bucket_cap(lim);
  uint64_t* dstp = row_pairs(a, sc, row_id);
  for (int ci = 0; ci < kCellsPerWg; ++ci) {
    const int cellno = cell0 + ci;
    const int t_begin = cellno * sc.cell;
    if (t_begin >= lim) break;
    const int t_end = min(t_begin + sc.cell, lim);
    const int t0 = t_begin + 4 * tid;
    f32x4 svn = {0.f, 0.f, 0.f, 0.f};
    if (ci + 1 < kCellsPerWg) svn = load4(cellno + 1);
    // the counting atomic also ranks the pair inside its (cell, bucket) run
    int bk[4] = {0, 0, 0, 0};
    uint32_t rk[4] = {0, 0, 0, 0};
    if (t0 < t_end) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        bk[e] = bucket_of_score(spl, top, sv4[e]);
        rk[e] = atomicAdd(&cnt[bk[e]], 1u);
      }
    }
    __syncthreads();                            // also: the previous cell's staging has been written out
    if (tid < kNBMax) {                         // one wavefront: staging offsets and the claims
      const uint32_t v = cnt[tid];
      cnt[tid] = 0u;                            // for the next cell
      uint32_t incl = v;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const uint32_t u = __shfl_up(incl, o);
        if (tid >= o) incl += u;
      }
      const uint32_t excl = incl - v;
      cur[tid] = excl;
      uint32_t d = 0xffffffffu;
      if (v > 0) {
        const uint32_t at = atomicAdd(&sc.cursor[row_id * kNBMax + tid], v);
        if (at + v <= cap) d = (uint32_t)tid * cap + at - excl;
        else sc.rowflag[row_id] = 1u;
      }
      delta[tid] = d;
    }
    __syncthreads();
    if (t0 < t_end) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t slot = cur[bk[e]] + rk[e];
        if (slot < (uint32_t)kCellMax) {
          stage[slot] = sort_key(sv4[e], (uint32_t)(t0 + e));
          const uint32_t d = delta[bk[e]];
          sdst[slot] = d == 0xffffffffu ? d : d + slot;
        } else {
          raise(a, sc, 1u);
        }
      }
    }
    __syncthreads();
    const int n_here = t_end - t_begin;
    for (int i = tid; i < n_here; i += kScatterThreads) {
      const uint32_t d = sdst[i];
      if (d != 0xffffffffu) dstp[d] = stage[i];
    }
    sv4 = svn;
  }
}

// Exact path, pass 3 (rows on the redo list): the same staging, destinations from the counted
// offsets; the row's pairs end up compact, in bucket order, from the start of its regions.
__global__ __launch_bounds__(256) void scatter_exact_kernel(PlanArgs a, Scratch sc, int64_t rows) {
  __shared__ __attribute__((aligned(16))) float spl[kNBMax];
  __shared__ uint32_t cur[kNBMax];              // next free staging slot of each bucket
  __shared__ uint32_t delta[kNBMax];            // global offset of the bucket's run - its first slot
  __shared__ uint64_t stage[kCellMax];
  __shared__ uint32_t sdst[kCellMax];
  const int64_t nredo = min((int64_t)sc.counters[3], rows);
  for (int64_t item = blockIdx.x; item < nredo * sc.maxch; item += gridDim.x) {
    const int64_t row_id = sc.redo[item / sc.maxch];
    const int cellno = (int)(item % sc.maxch);
    const int lim = (int)kv_row_len(row_id % a.N, a.S, a.L, a.non_causal);
    const int t_begin = cellno * sc.cell;
    if (t_begin >= lim) continue;
    const int t_end = min(t_begin + sc.cell, lim);
    const int tid = threadIdx.x;
    const int64_t cell = (row_id * sc.maxch + cellno) * kNBMax;
    const float* sk = (a.s_k ? a.s_k : sc.sk) + row_base(a, row_id);
    const int t0 = t_begin + 4 * tid;
    f32x4 sv4 = {0.f, 0.f, 0.f, 0.f};
    if (t0 < t_end) sv4 = *reinterpret_cast<const f32x4*>(sk + t0);
    __syncthreads();                            // the previous item's staging has been written out
    if (tid < kNBMax) {                         // one wavefront: exclusive scan of the cell's counts
      spl[tid] = sc.splitters[row_id * kNBMax + tid];
      const uint32_t v = sc.chist[cell + tid];
      uint32_t incl = v;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const uint32_t u = __shfl_up(incl, o);
        if (tid >= o) incl += u;
      }
      cur[tid] = incl - v;
      delta[tid] = sc.coffs[cell + tid] - (incl - v);
    }
    __syncthreads();
    float top[7];
#pragma unroll
    for (int k = 0; k < 7; ++k) top[k] = spl[8 * k + 7];
    if (t0 < t_end) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float sv = sv4[e];
        const int bk = bucket_of_score(spl, top, sv);
        const uint32_t slot = atomicAdd(&cur[bk], 1u);
        if (slot < (uint32_t)kCellMax) {
          stage[slot] = sort_key(sv, (uint32_t)(t0 + e));
          sdst[slot] = delta[bk] + slot;
        } else {
          raise(a, sc, 1u);
        }
      }
    }
    __syncthreads();
    uint64_t* dstp = row_pairs(a, sc, row_id);
    const int n_here = t_end - t_begin;
    for (int i = tid; i < n_here; i += 256) {
      const uint32_t d = sdst[i];
      if (d < (uint32_t)lim) dstp[d] = stage[i];
      else raise(a, sc, 8u);
    }
  }
}


// Per prefix row: sort the sampled scores (descending) and keep every (ns / nb)-th one as a
// splitter; bucket k of the row then holds the scores s with exactly k splitters above s.
__global__ __launch_bounds__(256) void splitter_kernel(PlanArgs a, Scratch sc) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint64_t* keys = reinterpret_cast<uint64_t*>(smem);
  const int64_t row_id = blockIdx.x;
  const int n = (int)(row_id % a.N);
  float* out = sc.splitters + row_id * kNBMax;
  const int len = (int)kv_row_len(n, a.S, a.L, a.non_causal);
  const int nb = row_buckets(len);
  if (nb == 1) {
    if (threadIdx.x < kNBMax) out[threadIdx.x] = -INFINITY;
    return;
  }
  const int ns = len / kSampleStride;
  const int n2 = next_pow2(ns);
  const float* smp = sc.samples + row_id * (a.L / kSampleStride);
  for (int i = threadIdx.x; i < n2; i += 256) keys[i] = i < ns ? sort_key(smp[i], (uint32_t)i) : ~0ull;
  __syncthreads();
  bitonic_sort_lds(keys, n2, threadIdx.x, 256);
  if (threadIdx.x < kNBMax) {
    const int k = threadIdx.x + 1;     // splitter k separates buckets k-1 and k
    float v = -INFINITY;
    if (k < nb) v = ordered_to_float(~(uint32_t)(keys[(int64_t)k * ns / nb] >> 32));
    out[threadIdx.x] = v;
  }
}

// Span records handed to the sorts: (row, first rank, end rank, w).  w & 0xffff = first bucket
// of the span; w & kCompact: the row's pairs lie compact in rank order from the start of its
// regions (exact path), otherwise bucket k's pairs lie at k * bucket_cap from there and
// sc.bst[row][k] is the rank at which bucket k starts.
constexpr int kCompact = 0x10000;
// w & kFewBuckets: the span lies inside its first four buckets, whose first ranks are the second
// half of the record -- the sort then finds a pair's region without a trip to memory.
constexpr int kFewBuckets = 0x20000;

// Cuts a row's buckets (populations tot[0..nb)) into spans that fit the LDS sort and buckets
// that do not, and appends both lists to the global ones.  Called by thread 0 .. of a
// workgroup of at least kNBMax + 1 threads; bstart receives the ranks at which the buckets start.
__device__ inline void emit_spans(const PlanArgs& a, const Scratch& sc, int64_t row_id, int nb, int len,
                                  const uint32_t* tot, uint32_t* bstart, int layout, int2* lspan, int* lk0,
                                  int2* lbig, int* lbk, uint32_t* nsp, uint32_t* gbase) {
  if (threadIdx.x == 0) {
    uint32_t off = 0, span_begin = 0, ns = 0, nbig = 0;
    int span_k0 = 0;
    for (int k = 0; k < nb; ++k) {
      const uint32_t cnt = tot[k];
      bstart[k] = off;
      if (cnt > (uint32_t)kSpanCap) {
        if (off > span_begin) { lk0[ns] = span_k0; lspan[ns++] = make_int2((int)span_begin, (int)off); }
        lbk[nbig] = k;
        lbig[nbig++] = make_int2((int)off, (int)(off + cnt));
        span_begin = off + cnt;
        span_k0 = k + 1;
      } else if (off + cnt - span_begin > (uint32_t)kSpanCap) {
        lk0[ns] = span_k0;
        lspan[ns++] = make_int2((int)span_begin, (int)off);
        span_begin = off;
        span_k0 = k;
      }
      off += cnt;
    }
    bstart[nb] = off;
    if (off > span_begin) { lk0[ns] = span_k0; lspan[ns++] = make_int2((int)span_begin, (int)off); }
    if (off != (uint32_t)len) raise(a, sc, 2u);
    nsp[0] = ns; nsp[1] = nbig;
    // one reservation per list instead of one (slow, serialised) atomic per span
    gbase[0] = ns ? atomicAdd(&sc.counters[0], ns) : 0u;
    gbase[1] = nbig ? atomicAdd(&sc.counters[1], nbig) : 0u;
  }
  __syncthreads();
  if (threadIdx.x < nsp[0]) {
    if ((int64_t)(gbase[0] + threadIdx.x) < sc.max_spans) {
      const int k0 = lk0[threadIdx.x];
      const uint32_t q0 = bstart[min(k0, nb)], q1 = bstart[min(k0 + 1, nb)], q2 = bstart[min(k0 + 2, nb)],
                     q3 = bstart[min(k0 + 3, nb)], q4 = bstart[min(k0 + 4, nb)];
      const int few = (uint32_t)lspan[threadIdx.x].y <= q4 ? kFewBuckets : 0;
      sc.spans[2 * (gbase[0] + threadIdx.x)] =
          make_int4((int)row_id, lspan[threadIdx.x].x, lspan[threadIdx.x].y, k0 | layout | few);
      sc.spans[2 * (gbase[0] + threadIdx.x) + 1] = make_int4((int)q0, (int)q1, (int)q2, (int)q3);
    } else {
      raise(a, sc, 4u);
    }
  }
  if (threadIdx.x < nsp[1]) {
    if ((int64_t)(gbase[1] + threadIdx.x) < sc.max_spans)
      sc.bigspans[gbase[1] + threadIdx.x] =
          make_int4((int)row_id, lbig[threadIdx.x].x, lbig[threadIdx.x].y, lbk[threadIdx.x] | layout);
    else raise(a, sc, 4u);
  }
  if (threadIdx.x <= (unsigned)nb) sc.bst[row_id * (kNBMax + 1) + threadIdx.x] = bstart[threadIdx.x];
}

// Per prefix row, after the scatter: the bucket populations are the final cursor values; cut
// them into spans, or put the row on the redo list if one of its buckets did not fit.
__global__ __launch_bounds__(2 * kNBMax) void span_kernel(PlanArgs a, Scratch sc) {
  __shared__ uint32_t tot[kNBMax];
  __shared__ uint32_t bstart[kNBMax + 1];
  __shared__ int2 lspan[kNBMax + 1], lbig[kNBMax];
  __shared__ int lk0[kNBMax + 1], lbk[kNBMax];
  __shared__ uint32_t nsp[2], gbase[2];
  const int64_t row_id = blockIdx.x;
  const int len = (int)kv_row_len(row_id % a.N, a.S, a.L, a.non_causal);
  if (len == 0) return;
  if (sc.rowflag[row_id]) {
    if (threadIdx.x == 0) sc.redo[atomicAdd(&sc.counters[3], 1u)] = (int32_t)row_id;
    return;
  }
  const int nb = row_buckets(len);
  if (threadIdx.x < kNBMax) tot[threadIdx.x] = (int)threadIdx.x < nb ? sc.cursor[row_id * kNBMax + threadIdx.x] : 0u;
  __syncthreads();
  emit_spans(a, sc, row_id, nb, len, tot, bstart, 0, lspan, lk0, lbig, lbk, nsp, gbase);
}

// Exact path, pass 2 (rows on the redo list): offsets of the (cell, bucket) runs in
// bucket-major order, and the row's spans.
__global__ __launch_bounds__(4 * kNBMax) void scan_exact_kernel(PlanArgs a, Scratch sc, int64_t rows) {
  __shared__ uint32_t part[4][kNBMax];   // counts of bucket b in chunk group q
  __shared__ uint32_t tot[kNBMax];
  __shared__ uint32_t bstart[kNBMax + 1];
  __shared__ int2 lspan[kNBMax + 1], lbig[kNBMax];
  __shared__ int lk0[kNBMax + 1], lbk[kNBMax];
  __shared__ uint32_t nsp[2], gbase[2];
  const int64_t nredo = min((int64_t)sc.counters[3], rows);
  for (int64_t item = blockIdx.x; item < nredo; item += gridDim.x) {
    const int64_t row_id = sc.redo[item];
    const int len = (int)kv_row_len(row_id % a.N, a.S, a.L, a.non_causal);
    const int b = threadIdx.x % kNBMax, q = threadIdx.x / kNBMax;
    const int nb = row_buckets(len);
    const int nch = (len + sc.cell - 1) / sc.cell;
    const int c0 = (nch * q) / 4, c1 = (nch * (q + 1)) / 4;   // this thread's chunk range
    const uint16_t* ch = sc.chist + row_id * sc.maxch * kNBMax;
    uint32_t* co = sc.coffs + row_id * sc.maxch * kNBMax;
    uint32_t t = 0;
    if (b < nb)
      for (int c = c0; c < c1; ++c) t += ch[c * kNBMax + b];
    __syncthreads();                     // the previous row's tables are no longer read
    part[q][b] = t;
    __syncthreads();
    if (q == 0) tot[b] = part[0][b] + part[1][b] + part[2][b] + part[3][b];
    __syncthreads();
    emit_spans(a, sc, row_id, nb, len, tot, bstart, kCompact, lspan, lk0, lbig, lbk, nsp, gbase);
    __syncthreads();
    if (b < nb) {
      uint32_t running = bstart[b];
      for (int k = 0; k < q; ++k) running += part[k][b];
      for (int c = c0; c < c1; ++c) {
        co[c * kNBMax + b] = running;
        running += ch[c * kNBMax + b];
      }
    }
  }
}

constexpr int kSortThreads = 256;
constexpr int kPerThread = kSubBuckets / kSortThreads;   // sub-bucket counters scanned per thread

__global__ __launch_bounds__(kSortThreads) void span_sort_kernel(PlanArgs a, Scratch sc) {
  __shared__ uint64_t keys[kSpanCap];           // the span's keys grouped by sub-bucket (fallback: as loaded)
  static_assert((kSpanCap & (kSpanCap - 1)) == 0, "the fallback pads a span to a power of two in place");
  __shared__ uint32_t start[kSubBuckets + 1];
  __shared__ uint32_t fill[kSubBuckets];
  __shared__ uint32_t wsum[kSortThreads / 64];
  __shared__ uint32_t red[3];          // min / max of the ordered score bits, fullest sub-bucket
  const int tid = threadIdx.x;
  const uint32_t nspans = min(sc.counters[0], (uint32_t)sc.max_spans);
  // A workgroup sorts spans blockIdx.x, blockIdx.x + gridDim.x, ...  A thread keeps its (up to
  // kPerLoad) pairs of the span in registers until they are grouped, and requests the next
  // span's pairs as soon as those registers are free, while the current span is ranked.
  constexpr int kPerLoad = (kSpanCap + kSortThreads - 1) / kSortThreads;
  int4 sp = make_int4(0, 0, 0, 0);
  uint64_t held[kPerLoad];
  auto fetch = [&](uint32_t w) {
    sp = sc.spans[2 * w];
    const int4 sq = sc.spans[2 * w + 1];
    const int row_n = sp.x % a.N, row_zh = sp.x / a.N;
    const uint64_t* src = row_pairs(a, sc, row_zh, row_n);
    const int n = sp.z - sp.y;
    if (sp.w & kCompact) {
#pragma unroll
      for (int e = 0; e < kPerLoad; ++e) {
        const int i = tid + e * kSortThreads;
        held[e] = i < n ? src[sp.y + i] : 0ull;
      }
    } else {
      // rank r of the row lies in the bucket k with bst[k] <= r < bst[k+1], at slot r - bst[k]
      // of that bucket's region
      const uint32_t cap = bucket_cap(kv_row_len(row_n, a.S, a.L, a.non_causal));
      const int k0 = sp.w & 0xffff;
      if (sp.w & kFewBuckets) {
        // the span's first ranks per bucket came with the record; m = buckets after the first
        // that begin inside the span (uniform over the workgroup)
        const uint32_t q0 = (uint32_t)sq.x, q1 = (uint32_t)sq.y, q2 = (uint32_t)sq.z, q3 = (uint32_t)sq.w;
        const uint32_t end = (uint32_t)sp.z;
        const int m = (q1 < end ? 1 : 0) + (q2 < end ? 1 : 0) + (q3 < end ? 1 : 0);
        const uint32_t base0 = (uint32_t)k0 * cap - q0;
#pragma unroll
        for (int e = 0; e < kPerLoad; ++e) {
          const int i = tid + e * kSortThreads;
          uint64_t v = 0ull;
          if (i < n) {
            const uint32_t r = (uint32_t)(sp.y + i);
            uint32_t off = base0;                               // region start - first rank of the bucket
            if (m > 0 && r >= q1) off = (uint32_t)(k0 + 1) * cap - q1;
            if (m > 1 && r >= q2) off = (uint32_t)(k0 + 2) * cap - q2;
            if (m > 2 && r >= q3) off = (uint32_t)(k0 + 3) * cap - q3;
            v = src[off + r];
          }
          held[e] = v;
        }
      } else {                                  // many (nearly) empty buckets in one span
        const uint32_t* bst = sc.bst + (int64_t)sp.x * (kNBMax + 1);
        int k = k0;
        uint32_t b0 = bst[k], b1 = bst[k + 1];
#pragma unroll
        for (int e = 0; e < kPerLoad; ++e) {
          const int i = tid + e * kSortThreads;
          uint64_t v = 0ull;
          if (i < n) {
            const uint32_t r = (uint32_t)(sp.y + i);
            while (r >= b1) { ++k; b0 = b1; b1 = bst[k + 1]; }
            v = src[(uint32_t)k * cap + (r - b0)];
          }
          held[e] = v;
        }
      }
    }
  };
  if (blockIdx.x < nspans) fetch(blockIdx.x);
  for (uint32_t w = blockIdx.x; w < nspans; w += gridDim.x) {
    const int64_t base = row_base(a, sp.x / a.N, sp.x % a.N) + sp.y;
    const int len = sp.z - sp.y;
    const bool more = w + gridDim.x < nspans;
    if (tid == 0) { red[0] = 0xffffffffu; red[1] = 0u; red[2] = 0u; }
    for (int i = tid; i < kSubBuckets; i += kSortThreads) fill[i] = 0;
    uint32_t lo = 0xffffffffu, hi = 0u;
#pragma unroll
    for (int e = 0; e < kPerLoad; ++e) {
      if (tid + e * kSortThreads < len) {
        const uint32_t o = ~(uint32_t)(held[e] >> 32);   // ordered score bits (ascending = ascending score)
        lo = min(lo, o); hi = max(hi, o);
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      lo = min(lo, (uint32_t)__shfl_xor((int)lo, o));
      hi = max(hi, (uint32_t)__shfl_xor((int)hi, o));
    }
    __syncthreads();                              // red and fill are initialised
    if ((tid & 63) == 0) { atomicMin(&red[0], lo); atomicMax(&red[1], hi); }
    __syncthreads();
    const float flo = ordered_to_float(red[0]);
    const float fhi = ordered_to_float(red[1]);
    const float range = fhi - flo;
    const float scale = range > 0.f ? (float)kSubBuckets / range : 0.f;
    // fine bucket of a key: descending score -> ascending sub-bucket (monotone in the key)
    auto sub = [&](uint64_t k) {
      const float f = ordered_to_float(~(uint32_t)(k >> 32));
      return min(max((int)((fhi - f) * scale), 0), kSubBuckets - 1);
    };
    bool fallback = len < 64;
    if (!fallback) {
      int sb[kPerLoad];
#pragma unroll
      for (int e = 0; e < kPerLoad; ++e) {
        sb[e] = sub(held[e]);
        if (tid + e * kSortThreads < len) atomicAdd(&fill[sb[e]], 1u);
      }
      __syncthreads();
      // exclusive scan of the sub-bucket counts: kPerThread per thread, then across threads
      uint32_t cnt[kPerThread], run = 0, mx = 0;
#pragma unroll
      for (int e = 0; e < kPerThread; ++e) {
        cnt[e] = fill[kPerThread * tid + e]; run += cnt[e]; mx = max(mx, cnt[e]);
      }
      uint32_t incl = run;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const uint32_t v = __shfl_up(incl, o);
        if ((tid & 63) >= o) incl += v;
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, o));
      if ((tid & 63) == 63) wsum[tid >> 6] = incl;
      if ((tid & 63) == 0) atomicMax(&red[2], mx);
      __syncthreads();
      uint32_t woff = 0;
      for (int k = 0; k < (tid >> 6); ++k) woff += wsum[k];
      uint32_t ex = woff + incl - run;
#pragma unroll
      for (int e = 0; e < kPerThread; ++e) {
        start[kPerThread * tid + e] = ex; ex += cnt[e]; fill[kPerThread * tid + e] = 0;
      }
      if (tid == kSortThreads - 1) start[kSubBuckets] = ex;
      fallback = red[2] > (uint32_t)kSubMax;
      __syncthreads();
      if (!fallback) {
#pragma unroll
        for (int e = 0; e < kPerLoad; ++e)
          if (tid + e * kSortThreads < len) keys[start[sb[e]] + atomicAdd(&fill[sb[e]], 1u)] = held[e];
        if (more) fetch(w + gridDim.x);
        __syncthreads();
        // rank inside the sub-bucket by direct comparison
        for (int p = tid; p < len; p += kSortThreads) {
          const uint64_t k = keys[p];
          const int sbk = sub(k);
          const uint32_t s0 = start[sbk], s1 = start[sbk + 1];
          uint32_t rank = s0;
          for (uint32_t qd = s0; qd < s1; ++qd) rank += keys[qd] < k ? 1u : 0u;
          a.kv_perm[base + rank] = (int32_t)(uint32_t)k;
        }
      }
    }
    if (fallback) {
      const int n2 = next_pow2(len);
#pragma unroll
      for (int e = 0; e < kPerLoad; ++e) {
        const int i = tid + e * kSortThreads;
        if (i < n2) keys[i] = i < len ? held[e] : ~0ull;
      }
      if (more) fetch(w + gridDim.x);
      __syncthreads();
      bitonic_sort_lds(keys, n2, tid, kSortThreads);
      for (int i = tid; i < len; i += kSortThreads) a.kv_perm[base + i] = (int32_t)(uint32_t)keys[i];
    }
    __syncthreads();
  }
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
    // the bucket's pairs: at its rank in a compact row, else at the start of its region
    uint64_t* const home = row_pairs(a, sc, sp.x) +
        ((sp.w & kCompact) ? (int64_t)sp.y
                           : (int64_t)(sp.w & 0xffff) * bucket_cap(kv_row_len(sp.x % a.N, a.S, a.L, a.non_causal)));
    uint64_t* src = home;
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
    for (int i = tid; i < len; i += 256) a.kv_perm[base + i] = (int32_t)(uint32_t)home[i];
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------
hipError_t launch_plan(const PlanArgs& a, hipStream_t stream) {
  const Scratch sc = carve(a.scratch, a.Z, a.H, a.Hkv, a.L, a.S, a.non_causal);
  if (sc.total > a.scratch_bytes) return hipErrorInvalidValue;
  if ((int64_t)a.Z * a.H * a.N * sc.maxch > 0x7fffffff) return hipErrorInvalidValue;
  const int64_t rows = (int64_t)a.Z * a.H * a.N;
  const int G = a.H / a.Hkv;
  // dynamic LDS limits of the kernels that need more than the default
  constexpr size_t kScoreLds = (size_t)kSub * kKStride * 2;
  constexpr size_t kSplitterLdsMax = 128 * 1024;   // a row's sample (L / 64 scores, 8-byte keys) is sorted in LDS
  {
    static std::mutex mu;
    static uint64_t done = 0;
    const hipError_t se = once_per_device(mu, done, [] {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&pool_sq_sort_kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 8192 * 8 + 4 * kD * 4);
      if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&splitter_kernel),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSplitterLdsMax);
      return e;
    });
    if (se != hipSuccess) return se;
  }

  hipLaunchKernelGGL(init_kernel, dim3(1), dim3(64), 0, stream, sc, rows, a.status);
  hipLaunchKernelGGL(kguide_kernel, dim3(a.Z * a.Hkv * kGuideParts), dim3(256), 0, stream, a, sc);
  {
    int n2 = 1;
    while (n2 < a.S) n2 <<= 1;
    const size_t lds = (size_t)n2 * 8 + 4 * kD * 4;
    hipLaunchKernelGGL(pool_sq_sort_kernel, dim3((unsigned)rows), dim3(256), lds, stream, a, sc);
  }
  if (a.N > 1 || a.non_causal) {
    const int RB = (G * a.N + 31) / 32;
    const int RBG = (RB + kScoreWaves - 1) / kScoreWaves;
    const int nchunks = (a.L + sc.chunk - 1) / sc.chunk;
    const dim3 grid((unsigned)((int64_t)a.Z * a.Hkv * RBG * nchunks));
    hipLaunchKernelGGL(score_kernel, grid, dim3(64 * kScoreWaves), kScoreLds, stream, a, sc);
    {
      int ns2 = 1;
      while (ns2 < a.L / kSampleStride) ns2 <<= 1;
      if ((size_t)ns2 * 8 > kSplitterLdsMax) return hipErrorInvalidValue;   // unreachable: the API refuses L > 1M tokens
      hipLaunchKernelGGL(splitter_kernel, dim3((unsigned)rows), dim3(256), (size_t)ns2 * 8, stream, a, sc);
    }
    const dim3 cgrid((unsigned)(rows * ((sc.maxch + kCellsPerWg - 1) / kCellsPerWg)));
    hipLaunchKernelGGL(scatter_kernel, cgrid, dim3(kScatterThreads), 0, stream, a, sc);
    hipLaunchKernelGGL(span_kernel, dim3((unsigned)rows), dim3(2 * kNBMax), 0, stream, a, sc);
    // the exact path for rows in which a bucket outgrew its region: normally none, and these
    // three launches find an empty list
    const dim3 rgrid((unsigned)(rows * sc.maxch < kRedoGrid ? rows * sc.maxch : kRedoGrid));
    hipLaunchKernelGGL(count_kernel, rgrid, dim3(256), 0, stream, a, sc, rows);
    hipLaunchKernelGGL(scan_exact_kernel, dim3((unsigned)(rows < kRedoGrid ? rows : kRedoGrid)), dim3(4 * kNBMax), 0,
                       stream, a, sc, rows);
    hipLaunchKernelGGL(scatter_exact_kernel, rgrid, dim3(256), 0, stream, a, sc, rows);
    const int64_t sort_grid = sc.max_spans < 8192 ? sc.max_spans : 8192;
    hipLaunchKernelGGL(span_sort_kernel, dim3((unsigned)sort_grid), dim3(kSortThreads), 0, stream, a, sc);
    hipLaunchKernelGGL(big_sort_kernel, dim3(kBigGrid), dim3(256), 0, stream, a, sc);
  }
  return hipGetLastError();
}

}  // namespace s2o
