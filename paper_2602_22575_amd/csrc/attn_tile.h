// Per-wavefront building blocks shared by the three S2O attention kernels for gfx950
// (attention.hip: both passes in one launch; local.hip: own-segment pass, paper Alg. 2;
// prefix.hip: prefix walk, paper Alg. 3): one wavefront = 32 query rows against one
// 64-token key tile staged in LDS.
//
// MFMA formulation (v_mfma_f32_32x32x16_bf16), transposed so that a query row lives in one
// lane pair and softmax statistics need a single cross-lane step:
//   S^T[n, m] = sum_d K[n, d] Q[m, d]        A = K tile rows from LDS, B = Q from registers
//   O^T[d, m] = sum_n V^T[d, n] P^T[n, m]    A = V^T from LDS,        B = P from the S^T
//                                            accumulators (no data movement)
// Lane l = (m = l % 32, hh = l / 32).  A 32x32 accumulator block holds, in register i of lane
// l, the element [row 8*(i/4) + 4*hh + i%4][column m].  The B operand of the PV product takes
// registers 8*kk..8*kk+7 of an S^T block as its 8 contraction slots, so slot (hh, jj) is key
// 16*kk + 8*(jj/4) + 4*hh + jj%4 of the 32-key block.
//
// K and V tiles sit row-major (token rows of 256 bytes) in LDS, written there directly by
// global_load_lds (no staging registers): a wavefront instruction deposits 4 gathered rows
// as 1 KB, lane l at byte 16*l, so rows cannot be padded; bank conflicts are avoided by an XOR
// swizzle instead: the sixteen 16-byte chunks of row r are stored at slot chunk ^ swz(r)
// (each lane fetches, from global memory, the chunk that belongs at its LDS slot), with
// swz(r) = 4*(r%4) + 2*((r/4)%2) + (r/8)%2: the 16 rows a 16-byte K read touches land on 16
// different chunks, and the 4 rows x 64 bytes that half a wavefront touches in a transposing
// V read land on the four 16-bank groups.
// The K operand is a plain 16-byte read of a row; the V^T operand is read with the
// transposing LDS load ds_read_b64_tr_b16: within each group of 16 lanes, lane i receives
// element (i % 4) of the four 8-byte rows pointed to by lanes i/4, 4 + i/4, 8 + i/4 and
// 12 + i/4, so pointing lane r of a group at (key slot r/4, dims 4*(r%4)..+3) hands every
// lane the four keys of its contraction slots at its own head dimension.
//
// Online softmax: logits are kept in base-2 units (raw score * softmax_scale * log2 e).
// m_ref is the reference maximum the accumulated terms are expressed in; it follows the true
// running maximum lazily: terms are only rescaled when the maximum has grown by more than
// kLazy (2^8), so that in the common case a tile costs no pass over the accumulator.  Any
// reference gives the same result; tile masses and the stop test are ratios in one common
// reference.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace s2o {
namespace tile {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) i16x4 lds_i16x4;
typedef __attribute__((address_space(1))) void gvoid;
typedef __attribute__((address_space(3))) void lvoid;

constexpr int kD = 128;                  // head dim
constexpr int kBN = 64;                  // key tile
constexpr int kRowsPerWave = 32;         // query rows of one wavefront
constexpr int kRowElems = kD;            // K and V rows sit unpadded in LDS (256 B)
constexpr int kTileElems = kBN * kRowElems;
constexpr float kLazy = 8.0f;

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 t = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, t);
}

__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | (((r >> 2) & 1) << 1) | ((r >> 3) & 1); }

// Byte offset, inside its 256-byte global row, of the chunk that lane `lane` of a 4-row load
// instruction must fetch so that it lands at the right (swizzled) LDS slot; `row0` is the
// first of the 4 tile rows the instruction covers (lane l covers row row0 + l/16).
__device__ __forceinline__ int load_chunk_offset(int lane, int row0) {
  return 16 * ((lane & 15) ^ swz(row0 + (lane >> 4)));
}

// One 4-row load instruction: 64 lanes x 16 bytes from global memory straight into LDS.
__device__ __forceinline__ void load_rows_to_lds(const char* lane_src, uint16_t* lds_row0) {
  __builtin_amdgcn_global_load_lds((const gvoid*)lane_src, (lvoid*)lds_row0, 16, 0, 0);
}

// Per-lane element offsets of the MFMA operands inside a tile.
struct Operands {
  int koff[8];      // K operand: row 32*nb + m, chunk 2*kk + hh, for the 8 contraction steps
  int voff[4][2];   // V^T operand: [32-dim block][8-key half of a 16-key step]
  __device__ __forceinline__ void init(int lane) {
    const int m_ = lane & 31, hh = lane >> 5;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) koff[kk] = m_ * kRowElems + 8 * ((2 * kk + hh) ^ swz(m_));
    // lane (group g16 = lane/16, r = lane%16) points at key slot r/4 (+ 4 for the upper lane
    // half), dims 16*(g16&1) + 4*(r%4); the row's swizzle depends on the lane and on which
    // 8-key half of the 16-key step is read
    const int rl = ((lane & 15) >> 2) + 4 * (lane >> 5);
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int a8 = 0; a8 < 2; ++a8) {
        const int chunk = 4 * db + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
        voff[db][a8] = (rl + 8 * a8) * kRowElems + 8 * (chunk ^ swz(rl + 8 * a8)) + 4 * (lane & 1);
      }
  }
};

// Q fragments of a lane's row: dims 16*kk + 8*hh .. +8 for the 8 contraction steps.
__device__ __forceinline__ void load_q(const uint16_t* qrow, int hh, bf16x8 (&qf)[8]) {
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qrow + 16 * kk + 8 * hh);
}

// contraction slots (hh, jj): jj < 4 -> keys key0 + 4*hh + jj, jj >= 4 -> keys key0 + 8 + 4*hh + jj - 4
__device__ __forceinline__ bf16x8 read_vt(const uint16_t* vt, int key0, const int (&off)[2]) {
  const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(vt + key0 * kRowElems + off[0]));
  const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(vt + key0 * kRowElems + off[1]));
  const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
  const u32x4 w = {l2.x, l2.y, h2.x, h2.y};
  return __builtin_bit_cast(bf16x8, w);
}

// S^T = K Q^T for the key tile at `ks`
__device__ __forceinline__ void qk_tile(const uint16_t* ks, const Operands& op, const bf16x8 (&qf)[8],
                                        f32x16 (&s)[2]) {
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
      ka[pre][nb] = *reinterpret_cast<const bf16x8*>(ks + 32 * nb * kRowElems + op.koff[pre]);
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) {
    if (kk + 2 < 8) {
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
        ka[(kk + 2) % 3][nb] = *reinterpret_cast<const bf16x8*>(ks + 32 * nb * kRowElems + op.koff[kk + 2]);
    }
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
      s[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kk % 3][nb], qf[kk], s[nb], 0, 0, 0);
  }
}

// O^T += V^T P^T with the V tile at `vt`
__device__ __forceinline__ void pv_tile(const uint16_t* vt, const Operands& op, const bf16x8 (&pb)[4],
                                        f32x16 (&o)[4]) {
  // V^T fragments are fetched one contraction step (4 blocks of 32 dims) ahead
  bf16x8 va[2][4];
#pragma unroll
  for (int db = 0; db < 4; ++db) va[0][db] = read_vt(vt, 0, op.voff[db]);
#pragma unroll
  for (int st = 0; st < 4; ++st) {
    if (st + 1 < 4) {
#pragma unroll
      for (int db = 0; db < 4; ++db) va[(st + 1) & 1][db] = read_vt(vt, 16 * (st + 1), op.voff[db]);
    }
#pragma unroll
    for (int db = 0; db < 4; ++db)
      o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[st & 1][db], pb[st], o[db], 0, 0, 0);
  }
}

// ---------------------------------------------------------------------------------------
// Explicitly scheduled operand reads (used by local.hip and prefix.hip).
//
// The compiler cannot tell an LDS read of one tile buffer from the asynchronous global->LDS
// load that is filling another, so it drains every outstanding global load (s_waitcnt
// vmcnt(0)) before any LDS read it knows about: a tile fetch issued at the top of a step
// would be waited for at the step's first operand read, with the whole memory latency
// exposed.  The operand reads below are therefore issued from inline assembly, which the
// compiler's wait insertion does not look into, and every fragment is handed to its MFMA
// through an explicit `s_waitcnt lgkmcnt(n)` that names how many younger LDS reads may still be
// in flight (LDS reads complete in order).  The kernels wait for their own tile fetches
// themselves (wait_tile_loads) right before the barrier that publishes a tile.
//
// Addresses: one VGPR per fragment slot (the swizzle makes them lane-dependent), fixed for the
// whole kernel; tile buffer and sub-block are selected with the instruction's immediate offset.
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

__device__ __forceinline__ uint32_t lds_address(const void* p) { return (uint32_t)(uintptr_t)(lvoid*)p; }

template <int kOff>
__device__ __forceinline__ void lds_issue_b128(bf16x8& d, uint32_t addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(d) : "v"(addr), "n"(kOff) : "memory");
}
template <int kOff>
__device__ __forceinline__ void lds_issue_tr64(u32x2& d, uint32_t addr) {
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(d) : "v"(addr), "n"(kOff) : "memory");
}
// The same reads at address (addr ^ kXor): the XOR stays next to its read (a separate statement
// would be hoisted out of the loop and cost the register it was meant to save).
template <int kOff, int kXor>
__device__ __forceinline__ void lds_issue_b128_x2(bf16x8& d0, bf16x8& d1, uint32_t addr) {   // two reads, 32 rows apart
  if constexpr (kXor == 0) {
    asm volatile("ds_read_b128 %0, %2 offset:%3\n\tds_read_b128 %1, %2 offset:%4"
                 : "=&v"(d0), "=&v"(d1) : "v"(addr), "n"(kOff), "n"(kOff + kTileElems) : "memory");
  } else {
    uint32_t t;
    asm volatile("v_xor_b32 %2, %5, %3\n\tds_read_b128 %0, %2 offset:%4\n\tds_read_b128 %1, %2 offset:%6"
                 : "=&v"(d0), "=&v"(d1), "=&v"(t) : "v"(addr), "n"(kOff), "n"(kXor), "n"(kOff + kTileElems) : "memory");
  }
}
template <int kOff, int kXor>
__device__ __forceinline__ void lds_issue_tr64_x(u32x2& d, uint32_t addr) {
  if constexpr (kXor == 0) {
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(d) : "v"(addr), "n"(kOff) : "memory");
  } else {
    uint32_t t;
    asm volatile("v_xor_b32 %1, %4, %2\n\tds_read_b64_tr_b16 %0, %1 offset:%3"
                 : "=&v"(d), "=&v"(t) : "v"(addr), "n"(kOff), "n"(kXor) : "memory");
  }
}
// The named values are valid once at most kYounger LDS reads issued after them are outstanding.
template <int kYounger>
__device__ __forceinline__ void lds_wait(bf16x8& a, bf16x8& b) {
  asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "n"(kYounger));
}
template <int kYounger>
__device__ __forceinline__ void lds_wait(u32x2& a, u32x2& b) {
  asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "n"(kYounger));
}
// Small reads issued among the fragment reads (stop votes, token indices): issue now, claim
// when at most kYounger reads issued after them may still be in flight.
__device__ __forceinline__ void lds_issue_word4(u32x4& d, uint32_t addr) {
  asm volatile("ds_read_b128 %0, %1" : "=v"(d) : "v"(addr) : "memory");
}
__device__ __forceinline__ void lds_issue_word(uint32_t& d, uint32_t addr) {
  asm volatile("ds_read_b32 %0, %1" : "=v"(d) : "v"(addr) : "memory");
}
template <int kYounger>
__device__ __forceinline__ void lds_wait(u32x4& a) { asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(a) : "n"(kYounger)); }
template <int kYounger>
__device__ __forceinline__ void lds_wait(uint32_t& a) { asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(a) : "n"(kYounger)); }
// All global->LDS tile loads (and every other global load) of this wavefront have landed.
__device__ __forceinline__ void wait_tile_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// ... all but the kYoungest most recent vector-memory instructions of the wavefront (they complete in order)
template <int kYoungest>
__device__ __forceinline__ void wait_older_loads() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(kYoungest) : "memory"); }

// Byte addresses of a lane's operand fragments inside a tile that starts at LDS address `base`
// (a multiple of 256).  The swizzle is an XOR on the 16-byte chunk index, i.e. on address bits
// 4..7, so the eight K slots and the second V half follow from one address each by an XOR
// with a constant: K step kk = k[0] ^ (kk << 5); V half 1 = (v[db] ^ 16) + 8 rows.  All sixteen
// are kept: an XOR at the point of use sits between the read and the MFMA that waits for it
// (12 XORs fewer per key tile for the V halves alone were worth 2 % of the walk).
struct OperandAddr {
  uint32_t k[8];      // K operand of contraction step kk, key block 0 (block 1: + 32 rows)
  uint32_t v[4];      // V^T operand: [32-dim block], keys 0..7 of a 16-key step (next step: + 16 rows)
  uint32_t vx[4];     // v[db] ^ 16: keys 8..15 of the step sit 8 rows on from there (saves an XOR per read)
  __device__ __forceinline__ void init(int lane, uint32_t base) {
    Operands op;
    op.init(lane);
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) k[kk] = (base + 2u * (uint32_t)op.koff[0]) ^ (uint32_t)(kk << 5);
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      v[db] = base + 2u * (uint32_t)op.voff[db][0];
      vx[db] = v[db] ^ 16u;
    }
  }
  // the same fragments in a tile kb / vb bytes further on (multiples of 256; may be "negative")
  __device__ __forceinline__ void shift(uint32_t kb, uint32_t vb) {
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) k[kk] += kb;
#pragma unroll
    for (int db = 0; db < 4; ++db) { v[db] += vb; vx[db] += vb; }
  }
  __device__ __forceinline__ OperandAddr at(uint32_t kb, uint32_t vb) const {
    OperandAddr r = *this;
    r.shift(kb, vb);
    return r;
  }
};

constexpr int kTileBytes = kTileElems * 2;          // 16 KB
constexpr int kHalfTileBytes = kTileBytes / 2;      // key block 1 of a K tile
constexpr int kVStepBytes = 16 * kRowElems * 2;     // one 16-key contraction step of a V tile

// The 16 K-fragment reads and 32 V^T-fragment reads of one step form one issue sequence
// (K read r = 2*kk + nb, then V read 16 + 2*(4*st + db) + half), so that the first V fragments
// are already on their way while the last score MFMAs run:
//   the K reads of kk = 0..kKAhead-1 up front; after the MFMAs of step kk the K reads of step
//   kk + kKAhead, or, once those are exhausted, the reads of two V fragments; the PV product
//   starts by requesting the rest of the first kVAhead V fragments and then, after the MFMA
//   of fragment c = 4*st + db, requests fragment c + kVAhead.
constexpr int kKAhead = 3;     // contraction steps of K fragments in flight (2 fragments each)
constexpr int kVAhead = 6;     // V fragments in flight (2 transposing reads each)
constexpr int kVEarly = 2 * kKAhead;   // V fragments requested during the score MFMAs

// LDS reads issued before the score MFMAs of step kk wait for their fragments
constexpr int issued_at_qk(int kk, bool with_v) {
  const int k_reads = 2 * (kk + kKAhead < 8 ? kk + kKAhead : 8);
  const int v_frags = with_v && kk + kKAhead > 8 ? 2 * (kk + kKAhead - 8) : 0;
  return k_reads + 2 * v_frags;
}

template <int kVOff, int c>
__device__ __forceinline__ void issue_v_fragment(const OperandAddr& oa, u32x2 (&vf)[16][2]) {
  lds_issue_tr64_x<kVOff + (c / 4) * kVStepBytes, 0>(vf[c][0], oa.v[c % 4]);
  lds_issue_tr64_x<kVOff + (c / 4) * kVStepBytes + 8 * kRowElems * 2, 0>(vf[c][1], oa.vx[c % 4]);
}

// S^T = K Q^T for the K tile at byte offset kKOff from the addresses in `oa`.  kWithV: also
// start the V^T reads of fragments 0..kVEarly-1 of the V tile at byte offset kVOff.
// `pre()` runs once the first K reads are out and before the first MFMA waits for them;
// `mid(kk)` after the MFMAs of contraction step kk have been handed over: work that only issues
// (LDS reads of its own, tile fetches for the next step) goes there, under the matrix pipe's
// shadow.  LDS reads issued from the hooks make the fragment waits a little conservative
// (they count only the fragment reads), never wrong.
template <int kKOff, int kVOff, bool kWithV, class Pre, class Mid>
__device__ __forceinline__ void qk_tile_sched(const OperandAddr& oa, const bf16x8 (&qf)[8], f32x16 (&s)[2],
                                              u32x2 (&vf)[16][2], Pre&& pre, Mid&& mid) {
  bf16x8 ka[8][2];
  static_for<0, kKAhead>([&](auto kk_) {
    constexpr int kk = decltype(kk_)::value;
    lds_issue_b128_x2<kKOff, 0>(ka[kk][0], ka[kk][1], oa.k[kk]);
  });
  pre();
  static_for<0, 8>([&](auto kk_) {
    constexpr int kk = decltype(kk_)::value;
    lds_wait<issued_at_qk(kk, kWithV) - (2 * kk + 2)>(ka[kk][0], ka[kk][1]);
    if constexpr (kk == 0) {
      f32x16 z;
#pragma unroll
      for (int i = 0; i < 16; ++i) z[i] = 0.f;
      s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kk][0], qf[kk], z, 0, 0, 0);
      s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kk][1], qf[kk], z, 0, 0, 0);
    } else {
      s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kk][0], qf[kk], s[0], 0, 0, 0);
      s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kk][1], qf[kk], s[1], 0, 0, 0);
    }
    if constexpr (kk + kKAhead < 8) {
      lds_issue_b128_x2<kKOff, 0>(ka[kk + kKAhead][0], ka[kk + kKAhead][1], oa.k[kk + kKAhead]);
    } else if constexpr (kWithV) {
      issue_v_fragment<kVOff, 2 * (kk + kKAhead - 8)>(oa, vf);
      issue_v_fragment<kVOff, 2 * (kk + kKAhead - 8) + 1>(oa, vf);
    }
    mid(kk_);
  });
}
template <int kKOff, int kVOff, bool kWithV>
__device__ __forceinline__ void qk_tile_sched(const OperandAddr& oa, const bf16x8 (&qf)[8], f32x16 (&s)[2],
                                              u32x2 (&vf)[16][2]) {
  qk_tile_sched<kKOff, kVOff, kWithV>(oa, qf, s, vf, [] {}, [](auto) {});
}

// The V^T reads qk_tile_sched started are not going to be used: their target registers stay
// claimed until the data has arrived (an LDS read that lands later would overwrite whatever
// the registers had been given to).
__device__ __forceinline__ void abandon_v_fragments(u32x2 (&vf)[16][2]) {
  static_for<0, kVEarly>([&](auto c_) { lds_wait<0>(vf[decltype(c_)::value][0], vf[decltype(c_)::value][1]); });
}

// O^T accumulate step with the accumulator updated in place.  As a builtin the compiler is free
// to give the result a tuple of its own, and for the loop-carried 64-register accumulator it
// does: a copy of O^T (32 two-register moves) per key tile.  In assembly the operand is tied.
// The compiler then no longer sees an MFMA and inserts no wait states around it.  In front: an
// MFMA must not read a register in the two issue slots after a VALU instruction wrote it, and
// the compiler does place moves of the operands right before the statement -- hence the two
// idle slots.  Behind: the next MFMA on the same accumulator needs none; before anything else
// reads or writes the accumulator, mfma_settle() must have run.
__device__ __forceinline__ void mfma_acc(f32x16& acc, const bf16x8& a, const bf16x8& b) {
  asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma_settle(f32x16 (&o)[4]) {
  asm volatile("s_nop 15\n\ts_nop 3" : "+v"(o[0]), "+v"(o[1]), "+v"(o[2]), "+v"(o[3]));
}

// O^T += V^T P^T.  kEarly: fragments 0..kVEarly-1 were requested by qk_tile_sched.
template <int kVOff, bool kEarly>
__device__ __forceinline__ void pv_tile_sched(const OperandAddr& oa, const bf16x8 (&pb)[4], f32x16 (&o)[4],
                                              u32x2 (&vf)[16][2]) {
  static_for<(kEarly ? kVEarly : 0), kVAhead>([&](auto c_) { issue_v_fragment<kVOff, decltype(c_)::value>(oa, vf); });
  static_for<0, 16>([&](auto c_) {
    constexpr int c = decltype(c_)::value, st = c / 4, db = c % 4;
    // V reads issued so far: fragments 0..kVAhead-1 and fragment c' + kVAhead after every earlier c'
    constexpr int frags = (c + kVAhead < 16 ? c + kVAhead : 16);
    lds_wait<2 * frags - (2 * c + 2)>(vf[c][0], vf[c][1]);
    const u32x4 w = {vf[c][0].x, vf[c][0].y, vf[c][1].x, vf[c][1].y};
    mfma_acc(o[db], __builtin_bit_cast(bf16x8, w), pb[st]);
    if constexpr (c + kVAhead < 16) issue_v_fragment<kVOff, c + kVAhead>(oa, vf);
  });
  mfma_settle(o);
}

// The same two products for a step that does them back to back (PV right after its scores).
template <int kKOff, class Pre, class Mid>
__device__ __forceinline__ void qk_tile_only(const OperandAddr& oa, const bf16x8 (&qf)[8], f32x16 (&s)[2], Pre&& pre,
                                             Mid&& mid) {
  u32x2 none[16][2];
  qk_tile_sched<kKOff, 0, false>(oa, qf, s, none, pre, mid);
}
template <int kKOff>
__device__ __forceinline__ void qk_tile_only(const OperandAddr& oa, const bf16x8 (&qf)[8], f32x16 (&s)[2]) {
  qk_tile_only<kKOff>(oa, qf, s, [] {}, [](auto) {});
}
template <int kVOff>
__device__ __forceinline__ void pv_tile_only(const OperandAddr& oa, const bf16x8 (&pb)[4], f32x16 (&o)[4]) {
  u32x2 vf[16][2];
  pv_tile_sched<kVOff, false>(oa, pb, o, vf);
}

// Value of the lane 32 away, combined with the lane's own (the two halves of a query row's
// statistics): v_permlane32_swap exchanges the upper half of one register with the lower half
// of another, so two copies of x come back as (x of lanes 0..31, x of lanes 32..63) in every
// lane -- no LDS round trip as with a bpermute.
__device__ __forceinline__ float xhalf_max(float x) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
}
__device__ __forceinline__ float xhalf_sum(float x) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r.x) + __uint_as_float(r.y);
}

// What a tile's score step hands to its PV step and to the row statistics.
struct TileStats {
  float alpha;   // factor that moves the old terms to the reference used for this tile (1 if unchanged)
  float mass;    // the tile's softmax mass for this lane's row, in that reference
  float prev;    // the row's mass so far, in that reference
  float m_use;   // the reference maximum used for this tile
  bool grow;     // the reference moved: the accumulator needs alpha
};

// Softmax numerators of a tile (left in s) and the row statistics.  kMask: apply the causal
// mask, the tile starting at key position key0 of the segment and the lane's row being qoff.
template <bool kMask>
__device__ __forceinline__ TileStats softmax_tile(f32x16 (&s)[2], float c2, float m_ref, float l_run, int key0,
                                                  int qoff, int hh) {
  float mx = -INFINITY;
#pragma unroll
  for (int nb = 0; nb < 2; ++nb)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if (kMask) {
        const int kpos = key0 + 32 * nb + 8 * (i >> 2) + 4 * hh + (i & 3);
        if (kpos > qoff) s[nb][i] = -INFINITY;     // CausalMask
      }
      mx = fmaxf(mx, s[nb][i]);
    }
  mx = xhalf_max(mx) * c2;
  TileStats t;
  t.grow = mx > m_ref + kLazy;
  t.m_use = t.grow ? mx : m_ref;
  float sum = 0.f;
  const float neg = -t.m_use;
#pragma unroll
  for (int nb = 0; nb < 2; ++nb)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float pe = __builtin_amdgcn_exp2f(fmaf(s[nb][i], c2, neg));
      s[nb][i] = pe;
      sum += pe;
    }
  sum = xhalf_sum(sum);
  t.mass = sum;
  t.alpha = t.grow ? __builtin_amdgcn_exp2f(m_ref - t.m_use) : 1.0f;
  t.prev = l_run * t.alpha;
  return t;
}

// The common tile of a ranked walk raises no row's maximum by much, and then the reference does
// not move: the numerators can be formed against the current reference straight away, without
// the pass that finds the tile's maximum first (17 instructions and a cross-lane exchange that
// the exponentials would have to wait for).  Whether that was admissible shows in the mass
// itself: a numerator is at most the mass, so a mass of at most kMassLimit bounds every bf16
// P value and every accumulator term by it.  `redo` (a larger mass, an overflow to infinity, or
// a row that has no reference yet) tells the caller to score the tile again and take
// softmax_tile.
constexpr float kMassLimit = 65536.0f;
__device__ __forceinline__ TileStats softmax_tile_keep_reference(f32x16 (&s)[2], float c2, float m_ref, float l_run,
                                                                 bool& redo) {
  TileStats t;
  t.grow = false;
  t.m_use = m_ref;
  t.alpha = 1.0f;
  t.prev = l_run;
  const float neg = -m_ref;
  float sum = 0.f;
#pragma unroll
  for (int nb = 0; nb < 2; ++nb)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float pe = __builtin_amdgcn_exp2f(fmaf(s[nb][i], c2, neg));
      s[nb][i] = pe;
      sum += pe;
    }
  t.mass = xhalf_sum(sum);
  redo = !(t.mass <= kMassLimit);
  return t;
}

// P^T fragments (bf16) for the four 16-key contraction steps
__device__ __forceinline__ void pack_p(const f32x16 (&s)[2], bf16x8 (&pb)[4]) {
#pragma unroll
  for (int st = 0; st < 4; ++st) {
    const int nb = st >> 1, k2 = st & 1;
    u32x4 w;
#pragma unroll
    for (int q = 0; q < 4; ++q) w[q] = pack_bf16x2(s[nb][8 * k2 + 2 * q], s[nb][8 * k2 + 2 * q + 1]);
    pb[st] = __builtin_bit_cast(bf16x8, w);
  }
}

// rare: move the accumulator to a new reference maximum (O^T *= alpha)
__device__ __forceinline__ void rescale(f32x16 (&o)[4], float al, bool gr) {
  if (__builtin_amdgcn_ballot_w64(gr) != 0ull) {
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        // in place: as plain C++ the products get registers of their own and the common path
        // (no rescale) pays for the merge with a copy of the whole accumulator per key tile
        float x = o[db][i];
        asm volatile("v_mul_f32 %0, %1, %0" : "+v"(x) : "v"(al));
        o[db][i] = x;
      }
  }
}

__device__ __forceinline__ void zero_acc(f32x16 (&o)[4]) {
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
}

// State buffers: a row's accumulator is kept as 128 fp32 = four 128-byte lines, one per 32-dim
// block db: the 16 values of the lane with hh = 0 in register order, then those of hh = 1
// (`sp` in load_acc = row base + 16*hh).
//
// lines_from_acc regroups the accumulators of a wavefront's 32 consecutive rows through two
// wavefront-private 4 KB LDS areas: afterwards lane L holds in o[db][4k .. 4k+3] the 16-byte
// piece L % 8 of line db of row 8k + L / 8, and a store instruction of store_acc_lines writes 8
// whole lines.  Stored straight from the accumulator layout an instruction would put 16 bytes
// into each of 64 lines: the same bytes in 16 times as many write requests, which is what the
// own-segment pass then waits for.  (LDS serves a wavefront's accesses in order: the reads
// behind the writes need no wait of their own.)
__device__ __forceinline__ void lines_from_acc(f32x16 (&o)[4], uint32_t area0, uint32_t area1, int lane) {
  // LDS accesses in assembly, like the fragment reads: the compiler would put a wait for every
  // outstanding global load in front of them (it cannot tell them from a global->LDS load's target)
  const int m_ = lane & 31, hh = lane >> 5, grp = lane >> 3, piece = lane & 7;
  const uint32_t wr = (uint32_t)(m_ * 128), rd = (uint32_t)(grp * 128 + ((piece ^ grp) << 4));
  uint32_t wq[4];                              // pieces rotated per row: no bank conflicts
#pragma unroll
  for (int q = 0; q < 4; ++q) wq[q] = wr + (uint32_t)(((hh * 4 + q) ^ (m_ & 7)) << 4);
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int db = 2 * pass + half;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const f32x4 v = {o[db][4 * q], o[db][4 * q + 1], o[db][4 * q + 2], o[db][4 * q + 3]};
        asm volatile("ds_write_b128 %0, %1" :: "v"((half ? area1 : area0) + wq[q]), "v"(v) : "memory");
      }
    }
    f32x4 r[2][4];
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int k = 0; k < 4; ++k)
        asm volatile("ds_read_b128 %0, %1" : "=v"(r[half][k]) : "v"((half ? area1 : area0) + rd + 1024u * k) : "memory");
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(r[0][0]), "+v"(r[0][1]), "+v"(r[0][2]), "+v"(r[0][3]), "+v"(r[1][0]), "+v"(r[1][1]),
                   "+v"(r[1][2]), "+v"(r[1][3])
                 :: "memory");
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int e = 0; e < 4; ++e) o[2 * pass + half][4 * k + e] = r[half][k][e];
  }
}
// `wave_rows` = the accumulator state of the wavefront's first row; o as left by lines_from_acc.
__device__ __forceinline__ void store_acc_lines(float* wave_rows, const f32x16 (&o)[4], int lane) {
  float* p = wave_rows + (lane >> 3) * kD + (lane & 7) * 4;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const f32x4 v = {o[db][4 * k], o[db][4 * k + 1], o[db][4 * k + 2], o[db][4 * k + 3]};
      *reinterpret_cast<f32x4*>(p + 8 * k * kD + 32 * db) = v;
    }
}
__device__ __forceinline__ void load_acc(const float* sp, f32x16 (&o)[4]) {
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(sp + 32 * db + 4 * i4);
      o[db][4 * i4] = v[0]; o[db][4 * i4 + 1] = v[1]; o[db][4 * i4 + 2] = v[2]; o[db][4 * i4 + 3] = v[3];
    }
}

// Normalise a wavefront's 32 output rows and store them as whole rows: the rows are regrouped
// through a wavefront-private 8 KB LDS area (32 rows x 256 bytes, the 16-byte chunks of a row
// rotated by the row number against bank conflicts), so that a store instruction writes 4
// complete rows (8 lines) where the accumulator layout would give 16 bytes to each of 32
// lines.  `tok` = the lane's destination row (a token index, the same in both lanes of a
// row); `head` + tok * row_stride is its address.
__device__ __forceinline__ void store_o_rows(uint16_t* head, int64_t row_stride, int tok, unsigned char* area,
                                             int lane, const f32x16 (&o)[4], float inv) {
  const int n = lane & 31, hh = lane >> 5;
  unsigned char* wr = area + n * 256 + 8 * hh;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {            // dims 32*db + 8*i4 + 4*hh + (0..3)
      u32x2 w;
      w.x = pack_bf16x2(o[db][4 * i4] * inv, o[db][4 * i4 + 1] * inv);
      w.y = pack_bf16x2(o[db][4 * i4 + 2] * inv, o[db][4 * i4 + 3] * inv);
      *reinterpret_cast<u32x2*>(wr + (((4 * db + i4) ^ (n & 15)) << 4)) = w;
    }
  const int sub = lane >> 4, chunk = lane & 15;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int row = 4 * k + sub;
    const u32x4 v = *reinterpret_cast<const u32x4*>(area + row * 256 + ((chunk ^ (row & 15)) << 4));
    const int t = __builtin_amdgcn_ds_bpermute(4 * row, tok);
    *reinterpret_cast<u32x4*>(head + (int64_t)t * row_stride + 8 * chunk) = v;
  }
}

// Normalise and store a lane's share of its output row: dims 32*db + 8*(i/4) + 4*hh + i%4.
__device__ __forceinline__ void store_o(uint16_t* orow, int hh, const f32x16 (&o)[4], float inv) {
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
      u32x2 w;
      w.x = pack_bf16x2(o[db][4 * i4] * inv, o[db][4 * i4 + 1] * inv);
      w.y = pack_bf16x2(o[db][4 * i4 + 2] * inv, o[db][4 * i4 + 3] * inv);
      *reinterpret_cast<u32x2*>(orow + 32 * db + 8 * i4 + 4 * hh) = w;
    }
}

// block id -> (head index z*H + h, segment counted from the last, position inside the
// segment's run of `per_seg` workgroups).  Longest prefixes first.  Consecutive block ids
// are dealt round-robin to the 8 XCDs, each with its own L2: the workgroups of one
// (z, h, segment) walk the same keys at about the same time, so they are given ids that land
// on one XCD (their K/V tiles then hit in that L2), while the XCD of a head rotates with the
// segment so that heads that stop early and heads that never stop mix evenly on every XCD.
__device__ __forceinline__ void map_block(int b, int ZH, int per_seg, int& zh, int& nr, int& pos) {
  if (ZH % 8 == 0) {
    const int xcd = b & 7, idx = b >> 3, per = ZH / 8;
    pos = idx % per_seg;
    const int unit = idx / per_seg;
    nr = unit / per;
    zh = ((xcd - nr) & 7) + 8 * (unit % per);
  } else {
    pos = b % per_seg;
    const int unit = b / per_seg;
    nr = unit / ZH;
    zh = unit % ZH;
  }
}

}  // namespace tile
}  // namespace s2o
