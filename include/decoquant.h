/*
 * decoquant.h - C ABI of libdecoquant: decode-step attention over a KV cache held in
 * DecoQuant form, and compression of newly appended K/V blocks, for AMD gfx950.
 *
 * Method: "DecoQuant" (arXiv 2405.12591).  A per-head block X[T_b, d] of keys or values is
 * regrouped as M[b1, (t, b2)] = X[t, b1*j2 + b2] (Preliminary, Eq. 2 with n = 2, i_1 = 1) and
 * factored exactly as M = T_S * T_L (Section 3.1, Eq. 3).  T_S (j1 x j1, carries the singular
 * values and the outliers) stays in fp16; T_L (j1 x T_b*j2, orthonormal rows, narrow range) is
 * quantized to `bits`-bit integers with one fp16 step per group (Preliminary, Eq. 1; Section
 * 3.1 "Local Tensor Quantization").  Decode attention reads the codes directly and applies
 * T_S by folding it into the query and into the P.V epilogue, which is the fusion of
 * dequantization with the product of the local tensors of Section 3.2 ("Kernel Fusion for
 * Dequantization") carried through the attention that follows it.
 *
 * Conventions for every entry point
 *   - All buffers are caller-owned DEVICE memory unless marked "host".  The library never
 *     allocates, frees or synchronises; all work is enqueued on the `hip_stream` argument
 *     (a hipStream_t passed as void*; NULL is the default stream).
 *   - fp16 values cross the boundary as uint16_t bit patterns (IEEE binary16).
 *   - Return value: DQ_OK (0) or a negative dq_status.  After DQ_EHIP, dq_last_hip_error()
 *     returns the hipError_t of the failed runtime call (as int).
 *   - Inputs are read-only.  Calls that share a workspace must be ordered on one stream.
 *
 * Storage layout of a compressed cache (B sequences, H kv heads, NB block slots per head;
 * tile = 128 tokens; c' = r*j2 + b2 is the element index inside a token row of T_L, r the
 * bond index, b2 the minor channel index; u = c + 2^(bits-1) is the stored field of code c):
 *   k_codes  u8   [B, H, NB, T_b, d*bits/8]   row t holds u of elements c' = 0..d-1, element e
 *                                             at bit (e*bits)%8 of byte (e*bits)/8
 *   k_scales f16  [B, H, NB, T_b, d/G]        step of group g = elements [g*G, (g+1)*G) of row t
 *   k_small  f16  [B, H, NB, j1, j1]          T_S of keys TRANSPOSED: entry [r][b1] = T_S[b1][r]
 *   v_codes  u8   [B, H, NB, T_b/128, j2, j1, 128*bits/8]
 *                                             for tile, b2, r: the 128 tokens of that tile,
 *                                             token tt at bit (tt*bits)%8 of byte (tt*bits)/8
 *   v_scales f16  [B, H, NB, T_b, d/G]        same grouping (by c') as keys
 *   v_small  f16  [B, H, NB, j1, j1]          T_S of values, entry [b1][r]
 * Token t of sequence b lives in block t / T_b, row t % T_b.
 *
 * Three local tensors (format field i3 = 8; Eq. 2 with n = 3, which Section 4.3 "Analysis of
 * Length of Local Tensors" reports as the more accurate, costlier variant): the row index is
 * factored as 1 * (T_b / 8) * 8 and the column index as j1 * j2 * 1,
 *   X[(a2, a3), (b1, b2)] = sum_{r, e} T_1[b1, r] T_2[r, a2, b2, e] T_3[e, a3],
 * T_1 = T_S as above, T_2 (orthonormal columns over (r, a2, b2)) is the quantized large tensor and
 * T_3 (8 x 8, fp16, carries the second cut's singular values) mixes the 8 tokens of a run of
 * consecutive tokens.  The codes and steps keep the layouts above with the bond index e in the
 * place of the token's low three bits (row a2*8 + e holds T_2[., a2, ., e]); two more arrays:
 *   k_small3 f16  [B, H, NB, 8, 8]            T_3 of keys TRANSPOSED: entry [a3][e] = T_3[e][a3]
 *   v_small3 f16  [B, H, NB, 8, 8]            T_3 of values, entry [e][a3]
 * A real token a2*8 + a3 then depends on all eight rows a2*8 + e: in the last, partly valid block
 * of a sequence every row of a run that contains a valid token must hold what dq_compress_kv
 * wrote (it writes whole blocks); runs wholly past seq_lens[b] may hold anything.
 *
 * A token factor on the small tensor (format field i1 = 2 or 4; Eq. 2 with n = 2 as printed, i_1 > 1):
 * the block's row index is factored as i1 * i2 (token t = a1*i2 + a2 of the block) and
 *   X[(a1, a2), (b1, b2)] = sum_r T_S[(a1, b1), r] T_L[r, (a2, b2)],   r = 0 .. i1*j1 - 1.
 * The large tensor keeps the block's shape: T_b rows of d elements, row a2*i1 + rho holding the
 * elements T_L[rho*j1 + r', (a2, b2)] at index r'*j2 + b2, with codes, steps and their layouts as
 * above (a "token row" is now one bond slice of one position a2).  The small tensors grow:
 *   k_small  f16  [B, H, NB, i1*j1, i1*j1]    entry [r][(a1, b1)] = T_S[(a1, b1)][r]  (transposed)
 *   v_small  f16  [B, H, NB, i1*j1, i1*j1]    entry [(a1, b1)][r]
 * A token then depends on rows all over its block: every row of a block that contains a valid
 * token must hold what dq_compress_kv wrote.  Decoding costs i1 times the multiply-adds; the plain
 * kernel serves these formats (the matrix-core kernel is built for i1 = 1).
 */
#ifndef DECOQUANT_H
#define DECOQUANT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum dq_status {
  DQ_OK = 0,
  DQ_EINVAL = -1,   /* null pointer, unsupported format, inconsistent sizes */
  DQ_ENOSPACE = -2, /* workspace smaller than dq_*_workspace_bytes() */
  DQ_EHIP = -3,     /* a HIP runtime call failed; see dq_last_hip_error() */
  DQ_ELIMIT = -4    /* dq_attn_decode_static: the sizes exceed what its built-in scratch memory holds */
} dq_status;

/* Format of a compressed cache.  Constraints: bits in {2, 4, 8}; head_dim == j1*j2;
 * head_dim in {64, 128}; j1 in {8, 16, 32}; group divides head_dim and group >= head_dim/2
 * or group divides head_dim/2; block_tokens is a positive multiple of 128; i3 in {1, 8};
 * levels in {0, 1}; i1 in {1, 2, 4} with i1 * j1 <= 32 and, for i1 > 1, i3 == 1. */
typedef struct dq_format {
  int32_t bits;         /* m of Eq. 1; qmax = 2^(m-1) - 1                         */
  int32_t group;        /* G: elements per step, consecutive inside one token row  */
  int32_t head_dim;     /* d                                                       */
  int32_t j1;           /* side of the small tensor T_S (Eq. 2: j_1)               */
  int32_t j2;           /* d / j1 (Eq. 2: j_2)                                     */
  int32_t block_tokens; /* T_b: tokens per decomposed block (Eq. 2: i_2; i_1 = 1)  */
  int32_t i3;           /* 1: two local tensors; 8: three, T_3 is 8 x 8 on the token side
                           (then i_2 = T_b / 8, i_3 = 8, j_3 = 1)                  */
  int32_t levels;       /* 0: the symmetric codes of Eq. 1, c in [-qmax, qmax];
                           1 (not the paper's): all 2^m codes, c in [-qmax - 1, qmax], with
                           step = fp16(max(max(x) / qmax, max(-x) / (qmax + 1))) so that neither
                           end clips.  Only the quantizer differs; decoding reads the stored
                           field c + 2^(m-1) the same way.                          */
  int32_t i1;           /* Eq. 2's i_1, the small tensor's share of the token index: 1 (the default
                           this library is built around), 2 or 4; then i_2 = T_b / i1, T_S is
                           (i1*j1) x (i1*j1) and mixes i1 groups of tokens as well as channels.
                           Needs i1*j1 <= 32 and i3 == 1.  See "A token factor" above.      */
} dq_format;

/* Device pointers to the arrays described above; shapes are fixed by (format, batch,
 * kv_heads, block_capacity).  k_small3 / v_small3 are read only when format.i3 == 8 (NULL
 * otherwise). */
typedef struct dq_cache {
  uint8_t* k_codes;
  uint16_t* k_scales;
  uint16_t* k_small;
  uint8_t* v_codes;
  uint16_t* v_scales;
  uint16_t* v_small;
  uint16_t* k_small3;
  uint16_t* v_small3;
  int32_t batch;
  int32_t kv_heads;
  int32_t block_capacity; /* NB */
} dq_cache;

/* Flags of dq_attn_decode. */
#define DQ_DECODE_AUTO 0u          /* fastest kernel that supports the format           */
#define DQ_DECODE_FORCE_GENERIC 1u /* scalar reference-grade HIP kernel, any format     */
#define DQ_DECODE_FORCE_MFMA 2u    /* matrix-core kernel; DQ_EINVAL if format unsupported */
/* Launch-shape overrides in the same word, for sweeps and tuning; a field of 0 leaves that choice to
 * the library, any other bit of the word is rejected with DQ_EINVAL.  They change how the work is
 * dealt to workgroups, never what is computed (results agree to the rounding of the partial sums). */
#define DQ_DECODE_SPLITS(n) (((uint32_t)(n) & 0x7Fu) << 8)       /* workgroups per (sequence, kv head): 1..64 */
#define DQ_DECODE_WAVES(n) (((uint32_t)(n) & 0xFu) << 16)        /* wavefronts per workgroup: 4 or 8 (matrix-core kernel) */
#define DQ_DECODE_UNIT_MAP(m) ((((uint32_t)(m) + 1u) & 0xFu) << 20) /* order of the units over the grid: 0..5 */

int32_t dq_version(void);
const char* dq_status_string(int32_t status);
int32_t dq_last_hip_error(void);

/* 1 if the matrix-core decode kernel supports (format, q_heads / kv_heads), else 0: head_dim 128,
 * j1 16, any code width, group 128 or 64.  One workgroup serves up to 4 (group 128) or 2 (group 64)
 * query heads of a kv head from one pass over its codes; more heads per kv head are served in head
 * groups of that many (the last one takes what is left: 7 = 4 + 3), each its own workgroup reading
 * the same codes (at most 16 groups).  Heads of 64 channels are also taken when j1 = j2 = 8,
 * group = 64, two local tensors, q_heads == kv_heads and kv_heads is even: two neighbouring kv
 * heads are then worked by one workgroup as one head of 128 channels. */
int32_t dq_decode_mfma_supported(const dq_format* fmt, int32_t q_heads, int32_t kv_heads);

/* Bytes of workspace dq_attn_decode needs for these sizes (0 on invalid arguments).  The
 * workspace holds split-sequence partial results; its first use must be preceded by one
 * dq_workspace_init() call (it contains counters the kernels leave at zero afterwards). */
size_t dq_decode_workspace_bytes(const dq_format* fmt, int32_t batch, int32_t q_heads,
                                 int32_t kv_heads, int32_t max_seq_len);

/* Zero-fill a workspace with a kernel (safe under stream capture). */
int32_t dq_workspace_init(void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Decode-step attention against the compressed cache (Section 3.2): for every sequence b and
 * query head h_q, out[b, h_q, :] = softmax_t(q[b, h_q] . K_hat[t] * scale) . V_hat, over the
 * tokens t < seq_lens[b] of kv head h_q / (q_heads / kv_heads), where K_hat and V_hat are the
 * dequantized blocks T_S16 * (step * code).  No intermediate rounding to fp16; fp32
 * accumulation; one final round-to-nearest-even to fp16.
 *   q         f16 [B, q_heads, d]; B * q_heads <= 2^24 (DQ_EINVAL beyond)
 *   seq_lens  i32 [B]; 0 <= seq_lens[b] <= max_seq_len; a sequence of length 0 yields zeros
 *   max_seq_len  host integer upper bound on seq_lens, <= block_capacity * T_b (sizes the grid)
 *   softmax_scale  <= 0 selects 1/sqrt(d)
 *   out       f16 [B, q_heads, d]
 *   out_f32   optional f32 [B, q_heads, d] copy of the result before the fp16 rounding, or NULL
 * Tokens >= seq_lens[b] are never used: their codes, steps and whole blocks may hold anything.
 */
int32_t dq_attn_decode(const dq_format* fmt, const dq_cache* cache, const uint16_t* q,
                       int32_t q_heads, const int32_t* seq_lens, int32_t max_seq_len,
                       float softmax_scale, uint16_t* out, float* out_f32, void* workspace,
                       size_t workspace_bytes, uint32_t flags, void* hip_stream);

/*
 * Same operation as dq_attn_decode, with two caller-created hipEvent_t handles that receive
 * the begin and end timestamps of the streaming kernel (the kernel that reads the codes).  For
 * measurement of that kernel's duration (Section 4.4 of the paper measures decode latency);
 * either handle may be NULL.
 */
int32_t dq_attn_decode_timed(const dq_format* fmt, const dq_cache* cache, const uint16_t* q,
                             int32_t q_heads, const int32_t* seq_lens, int32_t max_seq_len,
                             float softmax_scale, uint16_t* out, float* out_f32, void* workspace,
                             size_t workspace_bytes, uint32_t flags, void* hip_stream,
                             void* ev_kernel_start, void* ev_kernel_stop);

/*
 * The tokens generated since the last compression, still in fp16 (Section 3.2: new key/value rows
 * are buffered and DecoQuant runs only once a block's worth has accumulated).  They follow the
 * compressed tokens of their sequence.
 *   k_tail, v_tail  f16 [B, kv_heads, capacity, d]
 *   tail_lens       i32 [B] device, 0 <= tail_lens[b] <= capacity; capacity <= 1024 (host integer)
 */
typedef struct dq_tail {
  const uint16_t* k_tail;
  const uint16_t* v_tail;
  const int32_t* tail_lens;
  int32_t capacity;
} dq_tail;

/*
 * dq_attn_decode over the compressed tokens t < seq_lens[b] followed by the fp16 tail tokens:
 * one softmax over the union.  The tail becomes one more partial result of the merge (computed
 * inside the matrix-core kernel while its first codes are on their way; by a small kernel of its
 * own ahead of the plain kernel).  Rows >= tail_lens[b] are read but never used: they may hold
 * anything, but all `capacity` rows must be readable.  `tail` may be NULL (then this is
 * dq_attn_decode).
 */
int32_t dq_attn_decode_tail(const dq_format* fmt, const dq_cache* cache, const uint16_t* q,
                            int32_t q_heads, const int32_t* seq_lens, int32_t max_seq_len,
                            const dq_tail* tail, float softmax_scale, uint16_t* out, float* out_f32,
                            void* workspace, size_t workspace_bytes, uint32_t flags, void* hip_stream);

/*
 * dq_attn_decode_tail without a workspace argument, for callers that cannot allocate device memory
 * or have nowhere to keep a workspace: code under HIP graph capture, tight serving loops, harnesses
 * that forbid allocation.  The split partials and tickets live in a device array inside the library
 * (about 16.5 MiB per GPU the library is used on, held until the process ends); the call allocates
 * and frees nothing and needs no dq_workspace_init.  Same arguments, kernels and results (bit for
 * bit) as dq_attn_decode_tail (`tail` may be NULL), with these limits and rules:
 *   - batch * q_heads <= 512, else DQ_ELIMIT (nothing is launched);
 *   - the device that is current when the call is made must be the stream's device; the array's
 *     address on that device is looked up on the first call there;
 *   - all calls on one GPU share that GPU's array: calls must be ordered on one stream (or otherwise
 *     serialised); calls that overlap on one GPU race.
 */
int32_t dq_attn_decode_static(const dq_format* fmt, const dq_cache* cache, const uint16_t* q,
                              int32_t q_heads, const int32_t* seq_lens, int32_t max_seq_len,
                              const dq_tail* tail, float softmax_scale, uint16_t* out, float* out_f32,
                              uint32_t flags, void* hip_stream);

/* Bytes of workspace dq_compress_kv needs for n_blocks = B * H blocks of keys plus as many of
 * values (0 on invalid arguments). */
size_t dq_compress_workspace_bytes(const dq_format* fmt, int32_t batch, int32_t kv_heads);

/*
 * Compress one new block of keys and one of values per (sequence, kv head) and write them
 * into block slot blk_idx[b] of the cache (Section 3.2 "KV Cache Quantization": DecoQuant is
 * applied when a block of appended tokens has accumulated; Section 3.1 for the two steps).
 *   k_new, v_new  f16 [B, H, t_new, d], 1 <= t_new <= T_b (host integer)
 *   blk_idx       i32 [B] device, 0 <= blk_idx[b] < block_capacity; negative skips sequence b
 *   n_valid       i32 [B] device, rows >= n_valid[b] (and rows >= t_new) count as zero; may be NULL;
 *                 a sequence with no valid row is skipped like one with a negative blk_idx
 * The decomposition is an eigen-decomposition of the fp64 Gram matrix M M^T (j1 x j1) by
 * cyclic Jacobi rotations: T_S = U diag(sigma), T_L = diag(1/sigma) U^T M; directions with
 * sigma <= 1e-6 sigma_max are dropped (T_S column and T_L row zero).  T_S saturates to the
 * fp16 range; bit 0 of the int32 at workspace[0] is set if that happened in any block of this
 * call, cleared otherwise.  The int32 at workspace[4] receives the largest number of Jacobi
 * sweeps any block needed (diagnostic).  Workspace layout: a 256-byte header (those two words),
 * the fp32 large tensors [B*H*2, T_b, d] in token-major form (readable after the call: K block
 * of (b, h) at index 2*(b*H+h), V block next), then one status word per block.
 * The factors are not unique (signs, order of equal singular values): only their product and
 * the orthonormality of T_L's rows are defined.
 * With format.i3 == 8 a second cut follows: the 8 x 8 Gram matrix over the token index a3 of the
 * first cut's right factor is diagonalised the same way, T_3 = diag(sigma') V'^T goes to
 * k_small3 / v_small3 and the fp32 workspace rows are replaced by T_2 (row a2*8 + e) before they
 * are quantized; t_new < T_b and n_valid keep their meaning (missing rows are zero).
 */
int32_t dq_compress_kv(const dq_format* fmt, dq_cache* cache, const uint16_t* k_new,
                       const uint16_t* v_new, int32_t t_new, const int32_t* blk_idx,
                       const int32_t* n_valid, void* workspace, size_t workspace_bytes,
                       void* hip_stream);

/*
 * dq_compress_kv for a run of blocks per (sequence, kv head), as a prompt leaves it (Section 3.2:
 * the cache is quantized block by block; every block is decomposed on its own): t_new >= 1 rows,
 * cut into ceil(t_new / T_b) blocks of T_b rows, block j going to slot blk_idx[b] + j.  Same
 * arguments and results as dq_compress_kv, whose kernels it shares (a block's bits do not depend on
 * the call that wrote it), with these differences: the workspace holds the fp32 large tensors of
 * all blocks ([B*H*blocks*2, T_b, d], K block j of (b, h) at index 2*((b*H+h)*blocks + j)) and is
 * sized by dq_compress_blocks_workspace_bytes; a block whose slot falls outside the cache or none
 * of whose rows is valid (rows >= n_valid[b]) is not written.  At most 2^22 blocks per call, keys
 * and values counted apart.
 */
size_t dq_compress_blocks_workspace_bytes(const dq_format* fmt, int32_t batch, int32_t kv_heads,
                                          int32_t t_new);
int32_t dq_compress_kv_blocks(const dq_format* fmt, dq_cache* cache, const uint16_t* k_new,
                              const uint16_t* v_new, int32_t t_new, const int32_t* blk_idx,
                              const int32_t* n_valid, void* workspace, size_t workspace_bytes,
                              void* hip_stream);

/* Flags of dq_compress_kv_ex. */
#define DQ_COMPRESS_KEEP_LARGE 0u /* the fp32 large tensors are left in the workspace (as dq_compress_kv) */
#define DQ_COMPRESS_NO_LARGE 1u   /* the caller will not read them: the library may skip that hand-off */
#define DQ_COMPRESS_PLAIN 2u      /* use the plain vector-code decomposition kernel whatever the shape (for comparison) */
#define DQ_COMPRESS_WAVES(n) (((uint32_t)(n) & 0xFu) << 8) /* wavefronts per block of the tuned decomposition
                                     kernel: 1, 2 or 4; 0 leaves the choice to the library (for sweeps).  With three
                                     local tensors 1 selects the build that makes both cuts and quantizes in one
                                     launch (the library's choice above 512 blocks), 2 and 4 the three launches */

/*
 * dq_compress_kv_blocks with flags (t_new <= T_b makes it dq_compress_kv): for callers that do not
 * read the fp32 large tensors back, such as a serving loop that compresses a block whenever a
 * tail fills (Section 3.2).  With DQ_COMPRESS_NO_LARGE the large-tensor region of the workspace
 * holds nothing defined after the call; where the library supports it (two local tensors, at most
 * 1024 blocks per call, keys and values counted apart; head_dim 128 with j1 16 and group 128 or 64,
 * or head_dim 64 with j1 8, group 64 and an even number of kv heads) the
 * large tensor is quantized inside the decomposition kernel and never goes through memory.  Cache
 * contents and status words are the same bits either way.  The workspace is sized as before; its
 * first 256 bytes must be zero before the first call with this flag (dq_workspace_init on the
 * workspace, or on its first 256 bytes, does that) and are left so: they hold a counter of finished
 * blocks besides the status words.
 */
int32_t dq_compress_kv_ex(const dq_format* fmt, dq_cache* cache, const uint16_t* k_new,
                          const uint16_t* v_new, int32_t t_new, const int32_t* blk_idx,
                          const int32_t* n_valid, void* workspace, size_t workspace_bytes,
                          uint32_t flags, void* hip_stream);

/*
 * The cache policy of Section 3.2 ("KV Cache Quantization") with every decision on the device: new
 * key/value rows are buffered in fp16 (the tail), and a sequence's tail is compressed into its next
 * block slot as soon as it holds block_tokens rows.  The state below, all device memory owned by
 * the caller, together with the dq_cache is one layer's complete cache; the host keeps no mirror of
 * the lengths and reads nothing back, so a step (append, then decode) can be captured in a graph
 * and replayed across block boundaries.
 *   k_tail, v_tail  f16 [B, H, block_tokens, d]   rows not yet compressed (16-byte aligned)
 *   tail_lens       i32 [B]   rows in the tail, 0 <= tail_lens[b] < block_tokens between calls
 *   seq_lens        i32 [B]   compressed tokens, a multiple of block_tokens
 * Decoding over the whole cache is dq_attn_decode_tail (or dq_attn_decode_static) with seq_lens and
 * the tail {k_tail, v_tail, tail_lens, capacity = block_tokens}.  block_tokens <= 1024.
 */
typedef struct dq_kv_state {
  uint16_t* k_tail;
  uint16_t* v_tail;
  int32_t* tail_lens;
  int32_t* seq_lens;
} dq_kv_state;

/* Flags of dq_cache_append. */
#define DQ_APPEND_NO_COMPRESS 1u /* the caller knows that no tail can fill in this call (every tail length +
                                    n_rows < block_tokens): the compression launch is left out.  Should a
                                    tail fill all the same, bit 1 of the status word below is set, that tail
                                    stays full and the rows that do not fit are dropped. */

/* Bytes of workspace dq_cache_append needs (0 on invalid arguments): the workspace of dq_compress_kv
 * followed by four int32 per sequence.  It must be zeroed once before its first use
 * (dq_workspace_init) and belongs to the calls of one cache, ordered on one stream. */
size_t dq_cache_append_workspace_bytes(const dq_format* fmt, int32_t batch, int32_t kv_heads);

/*
 * Append rows to the sequences of a layer (Section 3.2: the rows a decoding step generates, or a
 * piece of a prompt): sequence b takes the first counts[b] of the n_rows rows given for it.
 *   k_rows, v_rows  f16 [B, H, n_rows, d], 1 <= n_rows <= block_tokens (host integer), 16-byte aligned
 *   counts          i32 [B] device, clamped to [0, n_rows]; NULL: every sequence takes all n_rows
 * Enqueues, on `hip_stream`: a copy of the rows that fit behind each tail's end, which also moves
 * the lengths; dq_compress_kv (fp32 large tensors not kept) of every tail that has reached
 * block_tokens rows into slot seq_lens[b] / block_tokens, after which seq_lens[b] has grown by
 * block_tokens; and, when n_rows > 1, a copy of the rows that did not fit to the start of the emptied
 * tail.  Sequences whose tail did not fill are skipped by the compression.  Status: the int32 at
 * byte 12 of the workspace gets bit 0 set (and keeps it) when a tail filled but the cache had no free
 * block slot; that tail then stays full and further rows for it are dropped.  Bytes 0..7 are the
 * status words of the last compression as dq_compress_kv documents them.
 */
int32_t dq_cache_append(const dq_format* fmt, dq_cache* cache, const dq_kv_state* state,
                        const uint16_t* k_rows, const uint16_t* v_rows, int32_t n_rows,
                        const int32_t* counts, void* workspace, size_t workspace_bytes, uint32_t flags,
                        void* hip_stream);

/*
 * Quantize and pack a caller-supplied large tensor (Preliminary, Eq. 1 per group; Section 3.1
 * step 2).  step = fp16(max|x| / qmax), the exact quotient rounded once, ties to even;
 * code = clamp(nearest integer of the exact x / step, ties to even, +-qmax); step == 0 gives
 * codes 0.  With format.levels == 1 the clamp is [-qmax - 1, qmax] and
 * step = fp16(max(max(x) / qmax, max(-x) / (qmax + 1))), each quotient rounded once.  Results are
 * bit-exact functions of the input.
 *   t_large  f32 [n_rows, d], token-major rows (element c' = r*j2 + b2); n_rows % 128 == 0
 *   value_layout  0: write key layout (codes [n_rows, d*bits/8]);
 *                 1: write value layout (codes [n_rows/128, j2, j1, 128*bits/8])
 *   codes, scales  outputs; scales f16 [n_rows, d/G] in both layouts
 */
int32_t dq_quantize_pack(const dq_format* fmt, const float* t_large, int64_t n_rows,
                         int32_t value_layout, uint8_t* codes, uint16_t* scales,
                         void* hip_stream);

/*
 * Measurement helper: read `bytes` (multiple of 16) from src with 128-bit loads and fold them
 * into sink[0..3] (u32) so the reads cannot be elided.  Gives the achievable read bandwidth
 * that the decode kernel's rate is compared with.
 */
int32_t dq_stream_read(const void* src, size_t bytes, uint32_t* sink, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* DECOQUANT_H */
