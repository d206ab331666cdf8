/*
 * fa.h - C boundary of the MI355X (gfx950) flash-attention forward library.
 *
 * One operation: for every batch b, head h and valid query row i < n_b
 *
 *     o[b,h,i,:] = sum_j softmax_j( scale * q[b,h,i,:].k[b,h,j,:] + mask(i,j) ) * v[b,h,j,:]
 *     lse[b,h,i] = ln sum_j exp( scale * q.k + mask )            (natural log)
 *
 * evaluated tile by tile with a running maximum and sum, so the n x n score
 * matrix never exists in memory (paper Sec. 2.2: the standard attention
 * softmax(QK^T/sqrt(d_k))V restructured by tiling and fusion into O(n) memory,
 * same result).  mask(i,j) is 0 for visible keys and -infinity otherwise; key j
 * is visible to query i when
 *     j < n_b                       key-padding mask (paper Eq. 1, read as exclusion;
 *                                   padding is the tail of each sequence), and
 *     i - L <= j <= i + R           for a local layer with window (L, R); global layers
 *                                   have L = R = -1 (paper Sec. 4.1.3, "ModernBERT
 *                                   Attention Mapping": local 63/64, global -1/-1).
 * The arguments mirror the paper's operator contract (Sec. 4.1.3: inputs
 * Q, K, V and a 1-D padding description, attributes scale, window_size_left,
 * window_size_right, execution on the caller's HIP stream, run-time dispatch on
 * head_dim 32 / 64 / 128).  fa_fwd and fa_fwd_bf16 describe the padding by sequence
 * lengths; fa_fwd_ex also accepts the operator's additive 1-D key bias (Eq. 1) and
 * can apply the model's rotary position embedding to q and k inside the call (Sec. 2.4).
 * Every call can be recorded into a HIP graph.
 *
 * Memory and layout
 *   q, k, v, o : DEVICE pointers, [batch, heads, max_len, head_dim] row-major
 *                (fa_fwd / fa_fwd_bf16); 16-bit elements (IEEE half or bfloat16);
 *                each 16-byte aligned.  fa_fwd_ex takes element strides instead.
 *   lse        : DEVICE pointer, float32 [batch, heads, max_len], or NULL to skip.
 *   seq_lens   : DEVICE pointer, int32 [batch], valid length n_b of each sequence,
 *                or NULL meaning n_b = max_len for all b.  Values are clamped into
 *                [0, max_len] by the kernel (they cannot be inspected on the host
 *                without a synchronisation).
 *   Rows i >= n_b (padding) and rows with no visible key: o = 0, lse = -infinity.
 *   Values stored in padded K/V/Q rows never influence valid rows, whatever
 *   their bit patterns.
 *
 * Ownership and ordering
 *   The caller owns every buffer.  The library allocates no device memory, never
 *   synchronises, never changes the current device.  Work is enqueued on `stream`
 *   (a hipStream_t passed as void*; NULL = the default stream) and the call
 *   returns immediately.  q, k, v are read-only; o and lse must not overlap them.
 *   Results are bitwise reproducible from run to run (no atomics).
 *
 * Errors
 *   0  success (work enqueued).
 *   <0 FA_ERR_*: an invalid argument, detected on the host before anything touches
 *      the device; nothing was enqueued.
 *   >0 the hipError_t returned by this call's own kernel launch (an error left behind
 *      by the caller's earlier HIP work is neither reported nor cleared).
 *   No exceptions, no aborts, nothing is printed.
 */
#ifndef FA_H
#define FA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FA_VERSION 400 /* major*10000 + minor*100 + patch */

enum {
  FA_OK = 0,
  FA_ERR_NULL_POINTER = -1,  /* q, k, v or o is NULL (or params is NULL)               */
  FA_ERR_BAD_SHAPE = -2,     /* batch, heads or max_len <= 0, or too large for a grid;
                                a row stride below head_dim; o strides under which two
                                output rows would overlap (zero, negative, interleaved) */
  FA_ERR_BAD_HEAD_DIM = -3,  /* head_dim not in the supported set {32, 64, 128}        */
  FA_ERR_BAD_SCALE = -4,     /* scale is NaN or infinite (0 and negatives are legal)   */
  FA_ERR_BAD_WINDOW = -5,    /* window == 0 (fa_fwd, fa_fwd_bf16 only: every pair of
                                window_left / window_right is legal for fa_fwd_ex)     */
  FA_ERR_MISALIGNED = -6,    /* a tensor pointer is not 16-byte aligned, or a stride
                                is not a multiple of 8 elements                        */
  FA_ERR_BAD_DTYPE = -7,     /* dtype is not FA_DTYPE_F16 / FA_DTYPE_BF16              */
  FA_ERR_BAD_STRUCT = -8,    /* fa_params.struct_size does not match this header       */
  FA_ERR_BAD_TUNING = -9,    /* unknown bits in fa_params.tuning                       */
  FA_ERR_SCRATCH = -10       /* fa_fwd_ex_static_scratch: the call would use more scratch
                                than FA_STATIC_SCRATCH_BYTES                           */
};

enum { FA_DTYPE_F16 = 0, FA_DTYPE_BF16 = 1 };

/*
 * fa_fwd: fp16 attention forward (the paper's kernel is fp16, Sec. 4.1.3 "HIP Kernel
 * and ORT Registration").
 *
 *   batch, heads, max_len, head_dim : tensor extents; head_dim is 32, 64 or 128 (the
 *            paper's operator dispatches on these three at run time, Sec. 4.1.3).
 *   scale  : multiplies q.k before the softmax (the operator's `scale` attribute;
 *            1/sqrt(head_dim) in the paper's models).  Applied in fp32 to the
 *            fp32-accumulated dot product.
 *   window : < 0  global layer (every valid key visible);
 *            W >= 1 local layer with a band of W keys: L = (W-1)/2, R = W/2
 *            (integer division), so W = 128 is the paper's 63 / 64;
 *            0 is rejected.
 */
int fa_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
           int batch, int heads, const int32_t* seq_lens, int max_len, int head_dim,
           float scale, int window, void* stream);

/* fa_fwd_bf16: identical contract with bfloat16 q, k, v, o. */
int fa_fwd_bf16(const void* q, const void* k, const void* v, void* o, float* lse,
                int batch, int heads, const int32_t* seq_lens, int max_len, int head_dim,
                float scale, int window, void* stream);

/*
 * fa_fwd_ex: superset entry point.  Separate left / right window extents (the
 * paper's window_size_left / window_size_right attributes: < 0 = unbounded on
 * that side), explicit element strides (so [batch, len, heads, dim] or a packed
 * QKV buffer can be passed without a transpose), an additive 1-D key bias, and a
 * tuning word.
 *
 * Strides are in ELEMENTS; the head_dim axis always has stride 1.  A stride
 * triple that is all zero selects the dense [batch, heads, max_len, head_dim]
 * layout.  Every stride must be a multiple of 8 elements.  lse is always dense
 * [batch, heads, max_len].
 */
typedef struct fa_params {
  uint32_t struct_size; /* = sizeof(fa_params) */
  int32_t dtype;        /* FA_DTYPE_* */
  const void* q;
  const void* k;
  const void* v;
  void* o;
  float* lse;              /* may be NULL */
  const int32_t* seq_lens; /* device int32[batch], may be NULL */
  int32_t batch, heads, max_len, head_dim;
  float scale;
  int32_t window_left;  /* < 0: unbounded */
  int32_t window_right; /* < 0: unbounded */
  int64_t q_strides[3]; /* batch, head, row */
  int64_t k_strides[3];
  int64_t v_strides[3];
  int64_t o_strides[3];
  void* stream;
  uint32_t tuning; /* 0 = library's choice; FA_TUNE_* bits force a kernel shape
                      (for benchmarking sweeps; results are identical up to
                      summation order) */
  /* Additive key bias, the operator's pad_bias input (paper Sec. 4.1.3, Eq. 1): DEVICE
     pointer to [batch, max_len] values of the SAME 16-bit type as q/k/v, or NULL.
     key_bias[b, j] is added to scale * q_i.k_j for every head and query (it is not
     multiplied by scale); -infinity excludes key j, so any key mask can be expressed,
     and the paper's -65504 on padded keys works as written.  It applies on top of
     seq_lens and the window.  2-byte alignment.  Global layers of head_dim 64 / 128
     and the resident local-layer kernel keep their pipelines (the bias enters through
     the score product's accumulator input); wider or one-sided windows, head_dim 32
     and scale == 0 take the general (masked) kernel. */
  const void* key_bias;
  int64_t key_bias_stride; /* elements between batch rows; 0 = max_len; >= max_len */
  /* Rotary position embedding of q and k inside the call (the paper's classifier uses rotary
     embeddings with a long-context frequency rescaling, Sec. 2.4; it gives neither formula nor
     constants, so the published definition is followed and the caller supplies the angles).
     rope_cos / rope_sin: DEVICE pointers to fp32 tables [max_len][rope_stride], entry [i][f] =
     cos / sin of the angle of token position i and frequency f < head_dim/2 (times any amplitude
     factor); both NULL = no rotation.  Row i of q and of k is rotated in pairs (f, f + head_dim/2):
         x'[f] = x[f] cos[i][f] - x[f + D/2] sin[i][f],  x'[f + D/2] = x[f + D/2] cos[i][f] + x[f] sin[i][f]
     in fp32 and rounded to the 16-bit storage type before the score product, exactly as if the
     caller had rotated the tensors itself; v is not rotated.  Tables are shared by all batch
     elements and heads.  16-byte alignment; rope_stride in floats, 0 = head_dim/2, else a
     multiple of 4 and >= head_dim/2.  The 32-row key-split shape and the 384 / 512-row and mixed
     shapes are not used with a rotation. */
  const float* rope_cos;
  const float* rope_sin;
  int64_t rope_stride;
  /* Optional DEVICE scratch the caller lends to the call (16-byte aligned), or NULL.  It is used in
     one case: a rotation on a GLOBAL layer (no window).  There the in-call rotation turns every K
     tile once per query tile; with at least fa_rope_scratch_bytes(...) of scratch a first kernel
     rotates q and k once into the scratch and the attention kernel (in any of its tile shapes)
     runs on the rotated copies: same bits, 8K tokens x 12 heads 0.27 -> 0.21 ms.  Too small a
     scratch, a local layer or no rotation: ignored.  The scratch may be reused as soon as the
     stream has passed the call; two calls that overlap in time must not share it. */
  void* scratch;
  size_t scratch_bytes;
} fa_params;

/* tuning word: bits 0-3 query rows per workgroup, bits 4-7 V-operand path,
   bits 8-11 workgroup-to-tile mapping, bits 12-15 window kernel. */
#define FA_TUNE_BM_AUTO 0x0u
#define FA_TUNE_BM_128 0x1u  /* 4 wavefronts x 32 query rows  */
#define FA_TUNE_BM_256 0x2u  /* head_dim 64 and 32: 4 wavefronts x 64 query rows; head_dim 128 global
                                layers: 8 wavefronts x 32 rows on one pair of K/V stages */
#define FA_TUNE_BM_32 0x3u   /* 32 query rows, the 4 wavefronts split the keys (global layers of
                                head_dim 64 without a key bias; ignored otherwise).  The library
                                picks it by itself when the call has at most 256 blocks of 32 query
                                rows (one per compute unit) and max_len > 128. */
#define FA_TUNE_BM_384 0x4u  /* 12 wavefronts x 32 query rows sharing one K/V stage (global layers of
                                head_dim 64 without a key bias; ignored otherwise) */
#define FA_TUNE_BM_512 0x5u  /* 8 wavefronts x 64 query rows sharing one K/V stage (same restriction) */
#define FA_TUNE_BM_MIXED 0x6u /* 256-row and 128-row workgroups in one launch, split on the device from
                                 the sequence length (same restriction, and batch 1, heads <= 256;
                                 ignored otherwise) */
#define FA_TUNE_V_AUTO 0x00u
#define FA_TUNE_V_LDS_TRANSPOSE 0x10u /* ds_read_b64_tr_b16 operand loads */
#define FA_TUNE_V_SCALAR 0x20u        /* 16-bit LDS reads (slow reference path) */
#define FA_TUNE_MAP_AUTO 0x000u
#define FA_TUNE_MAP_LINEAR 0x100u     /* workgroup id = tile id */
#define FA_TUNE_MAP_XCD 0x200u        /* tiles of one head kept on one XCD's L2 */

#define FA_TUNE_WIN_AUTO 0x0000u
#define FA_TUNE_WIN_PIPELINED 0x1000u /* local layers: never the two-phase kernel (K, then V, through one
                                         LDS region; four workgroups per compute unit), i.e. the
                                         pipelined kernels with K and V resident or in a ring */

#define FA_TUNE_WIN_TWO_PHASE 0x2000u /* local layers: the two-phase kernel wherever it applies (narrow two-sided
                                         windows), also on calls small enough to be latency-bound */

int fa_fwd_ex(const fa_params* params);

/*
 * Device scratch the library needs for a call of this shape, in bytes.  The
 * forward keeps all partial state in registers and LDS, so this is 0 for every
 * shape: the working set is the caller's O(n) tensors only.
 */
size_t fa_workspace_bytes(int batch, int heads, int max_len, int head_dim);

/* Bytes of fa_params.scratch with which a rotation on a global layer of this shape is done ahead
   of the attention kernel: rotated copies of q and k, 2 * batch * heads * max_len * head_dim * 2. */
size_t fa_rope_scratch_bytes(int batch, int heads, int max_len, int head_dim);

/*
 * fa_fwd_ex_static_scratch: fa_fwd_ex for callers that cannot allocate device memory and have
 * no scratch of their own to lend (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc).  params->scratch / scratch_bytes are ignored; where fa_fwd_ex would
 * use a lent scratch, this call uses an array of FA_STATIC_SCRATCH_BYTES that is part of the
 * library's device image (every GPU the library runs on holds its own copy from the first call
 * on it until the process ends).  A call that would need more returns FA_ERR_SCRATCH and
 * enqueues nothing; a call that would use no scratch behaves exactly like fa_fwd_ex.  It calls
 * no allocating routine.  All calls on one GPU share the one array: calls that overlap in time
 * on the same GPU (different streams, different threads) race on it; calls ordered on one
 * stream do not.  Nothing in the array needs to start at zero: every byte a call reads it has
 * written itself.  The first call on a GPU looks the array's address up (hipGetSymbolAddress);
 * make that call before a capture begins if the calls are to be recorded into a HIP graph.
 */
#define FA_STATIC_SCRATCH_BYTES (64u << 20)
int fa_fwd_ex_static_scratch(const fa_params* params);

/* Static, NUL-terminated description of a return code (FA_ERR_* or 0).  Positive
   codes map to a generic "HIP runtime error" string. */
const char* fa_strerror(int code);

/* FA_VERSION the library was built with. */
int fa_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FA_H */
