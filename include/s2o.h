/* s2o.h -- C ABI of the S2O causal prefill-attention library for AMD MI355X (gfx950).
 *
 * S2O ("early Stopping for Sparse attention via Online permutation") keeps Q/K/V where
 * they are in device memory and changes only which tokens are loaded in which order:
 *
 *   Step 1  s2o_plan       ranking (paper Sec. 3.1, Alg. 1, Eqs. (1)-(2)): per-segment mean
 *                          pooling of Q, a guide vector from the first key segment, a
 *                          token-level score for every query and every causal-prefix key,
 *                          and two Argsort-ed index maps (Q_perm, KV_perm).
 *   Step 2  s2o_attention  sparse attention (paper Sec. 3.2-3.3, Alg. 2-4): a dense causal
 *                          window inside each segment, then a FlashAttention-style walk
 *                          over the prefix in KV_perm order with gathered K/V rows, online
 *                          softmax and the monotone-gain early-stopping rule.
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer (hipMalloc'ed, or a torch CUDA tensor's
 *     data_ptr()); `params`, `out` and the size out-arguments are HOST pointers.
 *   - The library never allocates or frees device memory and never synchronises: a call
 *     validates its arguments on the host, enqueues kernels on `stream` (a hipStream_t
 *     passed as void*, NULL = the default stream) and returns.  The caller owns all
 *     buffers and keeps them alive until the stream has passed the call.  Because a call
 *     only enqueues kernels (no memset or copy nodes), it can be recorded into a HIP graph
 *     once it has run one time on the device outside a capture (the first call on a device
 *     sets kernel attributes).
 *   - Return value: S2O_OK (0) or a negative code.  On an argument error nothing is
 *     enqueued and nothing is written.
 *   - Tensors: Q [Z,H,L,D], K and V [Z,Hkv,L,D], O [Z,H,L,D]; bf16; the last dimension is
 *     contiguous; the other strides are given in elements (0 = packed default), multiples
 *     of 8.  One K or V head must span less than 4 GiB ((L-1) * row stride in bytes + 256
 *     < 2^32, row stride < 16 MiB; else S2O_EUNSUPPORTED).
 *     H % Hkv == 0 and query head h reads KV head h / (H/Hkv) (grouped-query attention).
 *   - Segments: N = L / S.  Packed prefix rows: for one (z,h) the KV_perm (and s_k) array
 *     has S*N*(N-1)/2 entries; row n (1 <= n < N, length n*S) starts at S*n*(n-1)/2.
 *     Segment 0 has no prefix.  (params.non_causal changes this: see s2o_params.)
 */
#ifndef S2O_H_
#define S2O_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define S2O_VERSION 4

enum {
  S2O_OK = 0,
  S2O_EINVAL = -1,        /* NULL pointer, bad struct_size, inconsistent shape/stride      */
  S2O_EUNSUPPORTED = -2,  /* valid request outside what the kernels implement              */
  S2O_ESCRATCH = -3,      /* scratch buffer missing, misaligned or too small               */
  S2O_EHIP = -4           /* a HIP runtime call failed; see s2o_last_hip_error()           */
};

typedef struct s2o_params {
  int32_t struct_size;   /* = sizeof(s2o_params)                                           */
  int32_t batch;         /* Z                                                              */
  int32_t q_heads;       /* H                                                              */
  int32_t kv_heads;      /* Hkv, H % Hkv == 0                                              */
  int32_t seq_len;       /* L, L % seg_len == 0                                            */
  int32_t head_dim;      /* D, only 128                                                    */
  int32_t seg_len;       /* S (paper default 2048), multiple of B_M; s2o_plan needs S <= 8192 */
  int32_t block_m;       /* B_M: query tile rows, 64 or 128                                */
  int32_t block_n;       /* B_N: key tile tokens, only 64                                  */
  int32_t use_q_perm;    /* 1: gather queries by Q_perm (Alg. 3); 0: original order (Alg. 4) */
  int32_t stop_mode;     /* 0: a triggering tile is discarded (Alg. 3/4 as printed);
                            1: it is folded in, then the walk stops (deferred check, App. A);
                            2: no stop rule is evaluated at all (App. A, kernel C)         */
  float softmax_scale;   /* 0 -> 1/sqrt(D)                                                 */
  int32_t max_prefix_tiles; /* 0: no budget; k > 0: a query tile visits at most the first k
                            tiles of its ranked prefix row (top-k selection, App. A)       */
  int32_t non_causal;    /* 0: causal prefill (the paper's setting).  1: every query attends
                            every key, as in the non-causal decomposition and top-k
                            comparisons of App. A: row n of KV_perm / s_K then ranks all L
                            tokens (rows of L entries, row n at n*L), there is no
                            own-segment pass and no state buffer, and every query row starts
                            its walk from the empty softmax state                          */
  int64_t q_stride[3];   /* element strides of Q for (z, h, l); all 0 -> packed [Z,H,L,D]  */
  int64_t k_stride[3];
  int64_t v_stride[3];
  int64_t o_stride[3];
} s2o_params;

/* Outputs of s2o_plan: caller-allocated device buffers.  q_perm and kv_perm are required;
 * the score outputs may be NULL (they exist so that the Argsort can be checked exactly
 * against the scores it sorted). */
typedef struct s2o_plan_out {
  int32_t* q_perm;   /* [Z,H,N,S]  segment-local offsets in [0,S), ordered by (s_q desc, offset asc) */
  int32_t* kv_perm;  /* [Z,H,S*N(N-1)/2] packed rows of absolute token indices < n*S,
                        ordered by (s_k desc, index asc); non_causal: [Z,H,N,L], indices < L */
  float* s_q;        /* [Z,H,N,S]  s_Q[n,s] = <Q[nS+s], k_guide>            (Eq. (1)), or NULL */
  float* s_k;        /* packed like kv_perm, indexed by token t (unsorted):
                        s_K[n,t] = <q_mean[n], K[t]>, t < n*S (non_causal: t < L)
                                                                            (Eq. (2)), or NULL */
  float* q_mean;     /* [Z,H,N,D]  segment means of Q, or NULL                             */
  float* k_guide;    /* [Z,Hkv,D]  mean of the first key segment, or NULL                  */
  int32_t* status;   /* one int32 (device), or NULL: 0 after a plan whose internal invariants all
                        held, else a mask of S2O_PLAN_* bits -- KV_perm is then not to be trusted.
                        The bits can only be set by a defect of the library or by NaN scores;
                        they exist so that such a plan cannot pass for a good one.           */
} s2o_plan_out;

/* bits of *s2o_plan_out.status */
enum {
  S2O_PLAN_STAGE_OVERFLOW = 1,  /* a bucket received more keys than were counted for it       */
  S2O_PLAN_COUNT_MISMATCH = 2,  /* a row's bucket counts do not add up to its length          */
  S2O_PLAN_SPAN_OVERFLOW = 4,   /* more sort spans than the scratch buffer has room for       */
  S2O_PLAN_BAD_RANK = 8         /* a key was ranked outside its row                           */
};

int s2o_version(void);
const char* s2o_strerror(int code);
/* hipError_t of the most recent failed HIP call made by this library on this thread. */
int s2o_last_hip_error(void);

/* Byte sizes of the s2o_plan outputs and of its scratch buffer (host only; any
 * out-pointer may be NULL). */
int s2o_plan_sizes(const s2o_params* params, size_t* q_perm_bytes, size_t* kv_perm_bytes,
                   size_t* s_q_bytes, size_t* s_k_bytes, size_t* q_mean_bytes,
                   size_t* k_guide_bytes, size_t* scratch_bytes);

/* Step 1 (Alg. 1).  Q, K: device bf16.  scratch: device, 256-byte aligned, at least the
 * size s2o_plan_sizes reports; contents are undefined afterwards.
 * Ties in either Argsort keep ascending index; -0 and +0 compare equal; NaN scores are an
 * input error (the maps are then permutations in an unspecified order). */
int s2o_plan(const void* Q, const void* K, const s2o_params* params, const s2o_plan_out* out,
             void* scratch, size_t scratch_bytes, void* stream);

/* s2o_plan for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the same ranking, with the scratch taken
 * from an array built into the library instead of a caller buffer.  The call allocates and
 * frees nothing (the array's address is looked up once per GPU, on the first call there).
 *   - Limit: configurations whose s2o_plan_sizes scratch_bytes exceed S2O_STATIC_SCRATCH_BYTES
 *     are refused with S2O_ESCRATCH before anything is enqueued (e.g. the Llama-3.1-8B head
 *     shape fits up to 8K tokens at S = 1024; 128K needs s2o_plan with a caller buffer).
 *   - Every GPU the library is loaded on holds the array until the process ends.
 *   - All calls on one GPU share that GPU's array: calls whose kernels may overlap (different
 *     streams, or other host threads) race; order them.  Contents do not survive the call; what
 *     the kernels need at zero is cleared by the call itself (by a kernel, so the call can be
 *     captured like s2o_plan).
 * Outputs and return codes as for s2o_plan. */
#define S2O_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
int s2o_plan_static(const void* Q, const void* K, const s2o_params* params, const s2o_plan_out* out,
                    void* stream);

/* Byte sizes of one counts array ([Z,H,L/B_M] int32) and of the optional attention scratch
 * (the per-row state buffers of the two-pass form, fp32 [Z,H,L,D+2]; 0 when non_causal). */
int s2o_attention_sizes(const s2o_params* params, size_t* counts_bytes, size_t* scratch_bytes);

/* Step 2 (Alg. 2 + Alg. 3, or Alg. 4 when use_q_perm == 0).
 *   q_perm   [Z,H,N,S] as produced by s2o_plan; ignored (may be NULL) if use_q_perm == 0.
 *   kv_perm  packed prefix rows; any permutation of [0, n*S) per row is legal (the maps
 *            need not come from s2o_plan).  Entries are clamped to [0, L), so a bad map cannot
 *            make the kernels read outside K and V, but a token >= n*S in the row of segment n
 *            would silently break causality.  Debug switch: with the environment variable
 *            S2O_VALIDATE_MAPS set (to anything but "0") every call that walks a prefix first
 *            checks on the device that all q_perm entries lie in [0, S) and all kv_perm
 *            entries of segment n in [0, n*S) ([0, L) when non_causal) and returns S2O_EINVAL
 *            otherwise; that check allocates a word of device memory and synchronises
 *            `stream`, so it is not for production loops or graph capture.
 *   tau      early-stop threshold.  Query tile j of segment n walks its prefix row in
 *            tiles of B_N tokens; with mass_i = sum over the tile of exp(x_it - m'_i) and
 *            prev_i = l_i * exp(m_i - m'_i) (the old normaliser in the new scale) the
 *            walk stops at the first tile where mass_i < tau * prev_i for every row i of
 *            the query tile.  tau <= 0 never stops and reproduces dense causal attention.
 *   O        [Z,H,L,D] bf16, rows in original order.
 *   computed [Z,H,L/B_M] prefix tiles folded into the output of permuted query tile
 *            n*(S/B_M)+j; skipped: prefix tiles never loaded.  n*S/B_N - computed - skipped
 *            is 1 when a triggering tile was loaded and discarded (stop_mode 0), else 0.
 *            Tiles beyond max_prefix_tiles count as skipped.  Either may be NULL.
 *            With non_causal the row of segment n lists L/B_N tiles (for every n, segment 0
 *            included), tau must be finite, scratch is ignored, and kv_perm may be NULL: every
 *            query tile then walks all keys in storage order without reading a map
 *            (contiguous dense attention, the decomposition's kernel A).
 *   scratch  NULL: one fused launch (the own-segment window and the prefix walk share
 *            registers).  Otherwise a device buffer, 256-byte aligned, of at least the size
 *            s2o_attention_sizes reports (else S2O_ESCRATCH): the call is then
 *            s2o_attention_local followed by s2o_attention_prefix on `stream`.  Both forms
 *            give the same result up to rounding order; the second does less own-segment work. */
int s2o_attention(const void* Q, const void* K, const void* V, const s2o_params* params,
                  const int32_t* q_perm, const int32_t* kv_perm, float tau, void* O,
                  int32_t* computed, int32_t* skipped, void* scratch, size_t scratch_bytes,
                  void* stream);

/* Pass 1 alone (Alg. 2): dense causal attention of every query over its own segment, queries
 * in original order, written as un-normalised online-softmax state into `scratch`
 * (required; the A / Lbuf / Mbuf buffers of the paper: per row (z,h,l) an fp32 accumulator
 * [D] in a kernel-private element order, the normaliser l and the reference maximum m in
 * base-2 logit units; layout: all accumulators, then all l, then all m).  It needs neither map,
 * so it may run before, or on another stream beside, s2o_plan. */
int s2o_attention_local(const void* Q, const void* K, const void* V, const s2o_params* params,
                        void* scratch, size_t scratch_bytes, void* stream);

/* Pass 2 alone (Alg. 3; Alg. 4's walk when use_q_perm == 0): resumes each row from the state
 * s2o_attention_local left in `scratch` (read only; the caller orders the two calls), walks
 * the prefix as described under s2o_attention, normalises and writes O and the counts.
 * With params.non_causal there is no state: scratch is ignored (may be NULL) and the call is
 * the same as s2o_attention; s2o_attention_local then returns S2O_EUNSUPPORTED. */
int s2o_attention_prefix(const void* Q, const void* K, const void* V, const s2o_params* params,
                         const int32_t* q_perm, const int32_t* kv_perm, float tau, void* O,
                         int32_t* computed, int32_t* skipped, const void* scratch, size_t scratch_bytes,
                         void* stream);

#ifdef __cplusplus
}
#endif
#endif /* S2O_H_ */
