/*
 * burst.h -- C ABI of the MI355X (gfx950) local-attention library.
 *
 * One device's share of a sequence-parallel attention ring (paper Sec. 2.2-2.4):
 * a resident query slice Q_i is attended against key/value chunks (K_j, V_j) that
 * arrive one at a time.  Each chunk's partial result is folded into a running
 * state (O_acc, m, l) by online softmax (paper Alg. 1); burst_finalize turns the
 * state into the output O_i and its log-sum-exp lse_i; the backward (paper Alg. 2)
 * recomputes the attention probabilities of a block pair from lse_i.
 *
 * Conventions common to every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  The library
 *     never frees caller memory and never synchronises the stream; every call
 *     only enqueues kernels on `stream` (a hipStream_t passed as void*, NULL =
 *     the default stream).  Pointers must be 16-byte aligned.
 *   - Tensors are indexed [B, H, rows, d] with d contiguous; per-row vectors
 *     (m, l, lse, D) are [B, H, rows].  fp32 tensors are always dense in that
 *     order; the tensors of type `dtype` are too unless burst_params.q_strides /
 *     kv_strides say otherwise.  K, V, dK, dV may have fewer heads than Q
 *     (burst_params.kv_heads; not in the paper).
 *   - Q, K, V, O, dO have element type `dtype` (bf16 or fp32).  The running
 *     state, lse, D and all gradients are fp32.
 *   - Scores are S = scale * Q K^T (Eq. 1 has scale = 1/sqrt(d); Alg. 1/2 omit
 *     it, here it is always applied).  scale must be finite and > 0.
 *   - Masking (not in the paper): with causal != 0 the key at global position
 *     k_off + c is visible to the query at global position q_off + r iff
 *     k_off + c <= q_off + r.  With window = w > 0 (paper Sec. 2.6: similarities
 *     a sparse pattern does not need are skipped) the key is visible only if
 *     k_off + c > q_off + r - w: a sliding window, the query itself and its w - 1
 *     predecessors when combined with causal; w = 0 means no window.  Key tiles and
 *     whole chunks outside the window are skipped, not computed and masked.
 *     With block_mask != NULL (block-sparse patterns, Sec. 2.6) a key must in addition
 *     lie in a block whose mask byte is nonzero; the three conditions are ANDed.  Key
 *     tiles no row of a workgroup can see are skipped.  The mask is read while the
 *     kernels run: keep it unchanged until they have finished.
 *     A row that sees no key keeps its state.
 *   - Return value: 0 on success, a negative burst_status otherwise.  On error
 *     nothing is enqueued and no output is written (entry points that enqueue
 *     several kernels check every kernel's limits before the first launch; only
 *     a launch failure reported by the HIP runtime itself, BURST_ERR_LAUNCH, can
 *     leave earlier kernels of the same call enqueued).
 *   - Thread safety: entry points may be called from several host threads.  The first
 *     call of a kernel family on a device sets that family's shared-memory function
 *     attributes (once per device, whichever thread comes first); that call cannot be
 *     recorded into a HIP graph, so run each entry point once eagerly on a device
 *     before capturing it.
 *   - Supported shapes: B, H >= 1; Nq, Nc >= 0 (0 = nothing to do); 1 <= d <= 128
 *     for the generic kernels; the bf16 MFMA kernels are used when dtype = bf16
 *     and d = 128.  Any Nq, Nc (ragged tails) are accepted.
 */
#ifndef BURST_H
#define BURST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum burst_dtype { BURST_BF16 = 0, BURST_F32 = 1 };

enum burst_status {
  BURST_OK = 0,
  BURST_ERR_NULL = -1,      /* a required pointer is NULL */
  BURST_ERR_ALIGN = -2,     /* a pointer is not 16-byte aligned */
  BURST_ERR_SHAPE = -3,     /* unsupported or inconsistent sizes, bad scale */
  BURST_ERR_DTYPE = -4,     /* unknown dtype */
  BURST_ERR_ARCH = -5,      /* current device is not gfx950 */
  BURST_ERR_LAUNCH = -6,    /* the HIP runtime reported a launch error */
  BURST_ERR_ALLOC = -7,     /* internal scratch allocation failed */
  BURST_ERR_TOO_LARGE = -8  /* burst_local_bwd_static: B*H*Nq > BURST_STATIC_MAX_ROWS */
};

typedef struct burst_params {
  int32_t B;        /* batch */
  int32_t H;        /* heads (the paper's Z) */
  int32_t Nq;       /* rows of the resident query slice (the paper's N/G) */
  int32_t Nc;       /* rows of this key/value chunk */
  int32_t d;        /* head dimension */
  int32_t dtype;    /* burst_dtype of Q, K, V, O, dO */
  int32_t causal;   /* 0 = every key visible, 1 = mask by global position */
  float   scale;    /* softmax scale, normally 1/sqrt(d) */
  int64_t q_off;    /* global position of query row 0 */
  int64_t k_off;    /* global position of row 0 of this chunk */
  int64_t window;   /* 0 = none; w > 0: keys at positions <= query position - w are hidden */
  const uint8_t* block_mask; /* NULL = none; else DEVICE pointer to a row-major byte matrix
                              * [ceil(Nq / block)][ceil(Nc / block)] for THIS query slice x chunk
                              * pair (one for all heads, or one per (batch, head), see
                              * block_mask_stride): entry (i, j) = 0 hides
                              * keys j*block .. of the chunk from query rows i*block .. of the slice */
  int32_t block;    /* edge of a mask block in rows = keys; a positive multiple of 64 when
                     * block_mask != NULL, ignored otherwise */
  int32_t kv_heads; /* 0 or H: K, V, dK, dV have H heads.  Otherwise (grouped-query attention) they
                     * have kv_heads heads, [B, kv_heads, Nc, d]; H must be a multiple of kv_heads and
                     * query head h uses key/value head h / (H / kv_heads); dK, dV sum over the group */
  int64_t block_mask_stride; /* bytes from one (batch, query head)'s flag matrix to the next, B*H
                     * matrices in all; 0 = one matrix shared by every batch entry and head */
  int64_t q_strides[3];  /* element strides {batch, head, row} of Q, dO and O (input and output);
                     * all zero = contiguous [B, H, Nq, d].  The last dimension is always contiguous.
                     * E.g. {Nq*H*d, d, H*d} addresses sequence-major [B, Nq, H, d] tensors (the
                     * layout of Sec. 2.2's backward messages) without a copy.  Row stride >= d, each
                     * stride a multiple of 16 bytes, none negative. */
  int64_t kv_strides[3]; /* the same for K_chunk and V_chunk ({batch, head, row}; kv_heads heads) */
} burst_params;

/* Alg. 1, initialisation: O_acc = 0, l = 0, m = -inf.
 * O_acc [B,H,Nq,d] fp32, m and l [B,H,Nq] fp32 (all written). */
int burst_state_init(float* O_acc, float* m, float* l, const burst_params* p, void* stream);

/* Alg. 1, body of the loop for one chunk, computed tile by tile (Sec. 2.4):
 * S = scale Q K_chunk^T (masked), per-row max / exp / sum, P V_chunk, and the
 * online-softmax merge into the state (m_new = max, rescale of l and O_acc).
 * Q [B,H,Nq,d], K_chunk and V_chunk [B,H,Nc,d] (read only); O_acc, m, l are
 * read and updated in place.  The state is any triple for which
 * m + log l and O_acc / l are the true log-sum-exp and output of the keys seen
 * so far; m is in natural-log units of the scaled scores and only a reference
 * point (it need not be the exact running maximum).  No S or P is ever stored. */
int burst_local_fwd(const void* Q, const void* K_chunk, const void* V_chunk,
                    float* O_acc, float* m, float* l, const burst_params* p, void* stream);

/* Alg. 1, last two steps: O = diag(l)^-1 O_acc (written as `dtype`),
 * lse = m + log l (fp32).  Rows with l = 0 give O = 0, lse = -inf. */
int burst_finalize(const float* O_acc, const float* m, const float* l,
                   void* O_out, float* lse, const burst_params* p, void* stream);

/* Alg. 1, the merge step on its own: state a <- merge(state a, state b), for
 * combining two partial walks over disjoint key sets (tree / multi-device
 * combine).  a is updated in place, b is read only. */
int burst_merge_state(float* O_a, float* m_a, float* l_a,
                      const float* O_b, const float* m_b, const float* l_b,
                      const burst_params* p, void* stream);

/* Alg. 2, pre-step: D = rowsum(dO o O).  O and dO [B,H,Nq,d] of `dtype`,
 * D [B,H,Nq] fp32 (written). */
int burst_bwd_prepare(const void* O, const void* dO, float* D, const burst_params* p, void* stream);

/* Alg. 2, one block pair (query slice x one chunk): recompute
 * S = scale Q K_chunk^T and P = exp(S - lse); dV += P^T dO; dP = dO V^T;
 * dS = P o (dP - D); dK += scale dS^T Q; dQ += scale dS K.
 * D may be NULL: it is then computed from O and dO into a scratch buffer that
 * the library owns, one per (device, stream), allocated with hipMalloc on the first
 * such call (and again when a later call needs a larger one: the old block is kept,
 * never freed, since enqueued kernels may still read it) and kept until process
 * exit.  Such a call therefore may allocate (never under stream capture: pass D
 * there), but it never frees or synchronises.  Calls with D == NULL are serialised
 * by a library lock from the buffer lookup to the last enqueue; consecutive calls
 * on one stream reuse the buffer in stream order.  With a non-NULL D nothing is
 * allocated or locked, O is not read and may be NULL.
 * dQ [B,H,Nq,d], dK_chunk and dV_chunk [B,H,Nc,d], all fp32.
 * accumulate_dq / accumulate_dkv: 1 = add to what the buffer holds (the caller
 * zero-fills before the first block pair), 0 = the buffer is overwritten with
 * this block pair's contribution.  Every output row is owned by one wavefront
 * (no atomics), so results are bitwise reproducible from run to run. */
int burst_local_bwd(const void* Q, const void* K_chunk, const void* V_chunk,
                    const void* O, const void* dO, const float* lse, const float* D,
                    float* dQ, float* dK_chunk, float* dV_chunk,
                    int accumulate_dq, int accumulate_dkv,
                    const burst_params* p, void* stream);

/* For callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, conventions and results as
 * burst_local_bwd with D == NULL (D = rowsum(dO o O) is computed by the call), except that D lives
 * in a static device array inside the library (BURST_STATIC_MAX_ROWS floats = 8 MiB per GPU, held
 * until the process ends) instead of an allocated buffer: this entry point calls no hipMalloc, no
 * hipFree and no allocating library routine, ever.  Its first call on a device looks up that
 * device's address of the array and sets the kernels' function attributes: run it once eagerly
 * on a device before capturing it.
 * Limit: B*H*Nq <= BURST_STATIC_MAX_ROWS, else BURST_ERR_TOO_LARGE (nothing enqueued).
 * All calls on one GPU share the array, which keeps the last call's D: nothing in it has to start
 * at zero (each call rewrites the B*H*Nq entries it reads), but two calls whose kernels can overlap
 * on one GPU (different streams without an event between them) race on it.  Calls on one stream,
 * from any number of host threads, are safe. */
#define BURST_STATIC_MAX_ROWS (2 * 1024 * 1024)
int burst_local_bwd_static(const void* Q, const void* K_chunk, const void* V_chunk,
                           const void* O, const void* dO, const float* lse,
                           float* dQ, float* dK_chunk, float* dV_chunk,
                           int accumulate_dq, int accumulate_dkv,
                           const burst_params* p, void* stream);

/* Size in bytes of the D buffer a burst_local_bwd call with these parameters and D == NULL needs
 * (B*H*Nq*4; the library's own buffer may be larger).  It is the only device memory the library
 * ever holds for a call: every other entry point, and burst_local_bwd with D given, is handed all
 * its buffers (the tiled steps keep S and P in registers, Sec. 2.4, and need no workspace).  A
 * caller that wants no library allocation allocates this many bytes, calls burst_bwd_prepare and
 * passes D.  Returns 0 for an invalid parameter block. */
size_t burst_workspace_bytes(const burst_params* p);

/* The two halves of burst_local_bwd on their own, for callers that need only one side
 * (Alg. 2 with the query side travelling needs dQ_j from every device but dK_i, dV_i only
 * locally) or that time them separately.  Same arguments and conventions as above; D must
 * be given.  burst_local_bwd(D != NULL) is exactly _dq followed by _dkv. */
int burst_local_bwd_dq(const void* Q, const void* K_chunk, const void* V_chunk,
                       const void* dO, const float* lse, const float* D,
                       float* dQ, int accumulate_dq, const burst_params* p, void* stream);
int burst_local_bwd_dkv(const void* Q, const void* K_chunk, const void* V_chunk,
                        const void* dO, const float* lse, const float* D,
                        float* dK_chunk, float* dV_chunk, int accumulate_dkv,
                        const burst_params* p, void* stream);

/* Alg. 1, body of the loop for one chunk exactly as printed, WITHOUT the tiling of
 * Sec. 2.4 (the "w/o LAO" variant of the paper's ablation, Tables 2-3): the whole
 * S_ij = scale Q K_chunk^T and P_ij = exp(S_ij - m_ij) of the block pair are stored in
 * `workspace` between the steps, then O_ij = P_ij V_chunk is merged into the state.
 * Same arguments, masking and resulting state as burst_local_fwd (up to rounding).
 * workspace: device memory, 256-byte aligned, at least
 * burst_materialized_workspace_bytes(p) bytes (B H Nq Nc (4 + element size) plus the
 * chunk's row statistics); owned by the caller, contents undefined afterwards except
 * that it starts with S_ij as fp32 [B,H,Nq,ceil8(Nc)] (raw scaled scores, unmasked),
 * followed at the next 256-byte boundary by P_ij in `dtype` with the same pitch
 * (masked entries and the padding columns are 0).  Returns BURST_ERR_SHAPE if
 * workspace_bytes is too small.  burst_materialized_workspace_bytes returns 0 for
 * invalid parameters. */
size_t burst_materialized_workspace_bytes(const burst_params* p);
int burst_local_fwd_materialized(const void* Q, const void* K_chunk, const void* V_chunk,
                                 float* O_acc, float* m, float* l,
                                 void* workspace, size_t workspace_bytes,
                                 const burst_params* p, void* stream);

/* Alg. 2, one block pair, in the same untiled form (the backward of the "w/o LAO" variant): the
 * seven steps of the loop body one after the other, S_ij, P_ij, dP_ij and dS_ij of the whole
 * block pair stored in `workspace` between them.  Same arguments, masking and results as
 * burst_local_bwd with D given (up to rounding).  workspace: device memory, 256-byte aligned,
 * at least burst_materialized_bwd_workspace_bytes(p) bytes (B H Nq Nc (4 + 2 element sizes));
 * afterwards it starts with dP_ij as fp32 [B,H,Nq,ceil8(Nc)], followed at the next 256-byte
 * boundaries by P_ij and dS_ij in `dtype` with the same pitch (hidden entries and padding 0;
 * dS_ij without the factor scale). */
size_t burst_materialized_bwd_workspace_bytes(const burst_params* p);
int burst_local_bwd_materialized(const void* Q, const void* K_chunk, const void* V_chunk,
                                 const void* dO, const float* lse, const float* D,
                                 float* dQ, float* dK_chunk, float* dV_chunk,
                                 int accumulate_dq, int accumulate_dkv,
                                 void* workspace, size_t workspace_bytes,
                                 const burst_params* p, void* stream);

/* For tests and tuning (no counterpart in the paper): which of the two kernel families serves
 * bf16, d = 128 calls.  0 = chosen per call (the default): forward and dQ from how well the call's
 * workgroups fill the chip and from the flags' block edge, dK/dV always hand-scheduled, with 64
 * instead of 128 keys per workgroup for 64-wide block flags; 1 = always the hand-scheduled kernels
 * (256 query rows, 128 keys per workgroup); 2 = always the plainly written ones (128 rows, 64 keys
 * per workgroup).  Process-wide; results of the two
 * families agree within the tolerance, not bitwise.  Returns BURST_ERR_SHAPE for another value. */
int burst_set_kernel_family(int family);
/* Which family would serve burst_local_fwd / the dQ half of burst_local_bwd for these parameters
 * under the current setting: 1 or 2 as above, 0 = neither (another head dimension or type, or a
 * shape only the generic kernels take); a negative burst_status for an invalid block.  Host
 * logic only, no device call. */
int burst_kernel_family_for(const burst_params* p);

/* Timing helper for harnesses that cannot create HIP events themselves:
 * records/queries events on the same stream the kernels are launched on.
 * burst_event_create returns an opaque handle (NULL on failure). */
void* burst_event_create(void);
int   burst_event_record(void* event, void* stream);
int   burst_event_elapsed_ms(void* start, void* stop, float* ms); /* waits for `stop` */
void  burst_event_destroy(void* event);

/* Micro-benchmarks for the measurement harness (no counterpart in the paper): the rates the
 * attention kernels are compared with, measured with the instruction forms they use.
 * burst_probe_mfma: 256 workgroups of 4 * wavefronts_per_simd (1 or 2) wavefronts; each wavefront
 * issues iters * 16 v_mfma_f32_32x32x16_bf16 (32768 FLOP each) and nothing else.  a_from_lds: 0 =
 * both operands stay in registers, 1 = the A operand of every MFMA is read fresh from LDS (128-bit
 * reads), 2 = of every second MFMA.  operands: 64 KiB of bf16 values on the device (their contents
 * set how many bits toggle, and with that the clock the chip sustains); sink: 256 * 512 floats,
 * written.  The caller times the launch.
 * burst_probe_atomic_dq: the memory traffic of a backward that would compute a block pair once,
 * keys stationary, and get its dQ partial sums out of the workgroups: heads * key_blocks workgroups
 * (heads a multiple of 8), each adding one [64][128] tile per 64 query rows into dQ [heads][Nq][128]
 * (Nq a multiple of 64).  mode 1: fp32 atomic adds; mode 0: plain stores in the same pattern; mode 2:
 * plain load-add-store in the same pattern (racing: timing only).  No arithmetic: a lower bound on
 * what such a kernel would take. */
int burst_probe_mfma(int a_from_lds, int wavefronts_per_simd, const void* operands, float* sink, int iters,
                     void* stream);
int burst_probe_atomic_dq(float* dQ, int heads, int Nq, int key_blocks, int mode, void* stream);

const char* burst_strerror(int status);
int         burst_version(void);

#ifdef __cplusplus
}
#endif
#endif /* BURST_H */
