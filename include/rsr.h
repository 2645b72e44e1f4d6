/*
 * librsr -- Redundant Segment Reduction (RSR) matrix-vector multiplication
 * for binary {0,1} and ternary {-1,0,+1} matrices on AMD MI355X (gfx950).
 *
 * C ABI.  Every pointer argument says whether it is a HOST or a DEVICE
 * pointer.  No function throws or aborts; failures are reported through
 * return codes and rsr_last_error().  The library is the product: there is no
 * CPU fallback, and every step listed below runs in HIP kernels.
 *
 * Orientation (paper, System Overview): the product is out = M * v with M of
 * shape rows x cols, v of length cols, out of length rows.  M is split into
 * horizontal blocks of k rows; inside a block, columns that carry the same
 * k-entry pattern are grouped, their entries of v are summed once, and every
 * group sum is distributed once to the block rows its pattern names.
 */
#ifndef RSR_H
#define RSR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rsr_handle_s *rsr_handle_t;

/* kind: what the handle holds */
enum {
    RSR_BINARY = 0,           /* M in {0,1}; one pass, 2^k patterns per block            */
    RSR_TERNARY_2PASS = 1,    /* M = M+ - M-, each half handled as a binary pass          */
    RSR_TERNARY_FUSED = 2,    /* one pass over base-3 patterns (3^k per block)            */
    RSR_DENSE_TERNARY_P2 = 3  /* comparison point: dense 2-bit packed ternary, no RSR     */
};

/* element type of the activation vector v */
enum { RSR_F32 = 0, RSR_BF16 = 1 };

/* error codes */
enum {
    RSR_OK = 0,
    RSR_EINVAL = 1,       /* null pointer, non-positive size, unknown enum, bad handle     */
    RSR_EVALUE = 2,       /* a matrix entry is outside the alphabet of the kind            */
    RSR_EUNSUPPORTED = 3, /* valid request outside the limits stated below                 */
    RSR_ENOMEM = 4,       /* device or host allocation failed                              */
    RSR_EHIP = 5,         /* a HIP runtime call failed                                     */
    RSR_EINTERNAL = 6,    /* a self-check of the preprocessing output failed               */
    RSR_ESCRATCH = 7      /* rsr_preprocess_into: the input needs more temporary memory    */
                          /* than the fixed scratch array (RSR_INTO_SCRATCH_BYTES)         */
};

/*
 * rsr_preprocess -- the one-time offline phase (paper, System Overview,
 * "Algorithm overview", and Kernels Implementation: counting sort over the
 * discrete pattern space, compact 16-bit metadata, indices ascending inside
 * a group, zero-contribution groups dropped).
 *
 *   M     DEVICE pointer, int8, row-major [rows][cols]; entries {0,1} for
 *         RSR_BINARY, {-1,0,+1} otherwise.  Borrowed: the caller keeps
 *         ownership and may free it as soon as the call returns.
 *   rows  number of outputs (>= 1); need not be a multiple of k (the last
 *         block is completed with zero rows, whose outputs are never written)
 *   cols  length of v, 1 <= cols <= 32766
 *   k     block height, or 0 to let the library choose (paper, Demonstration Scenarios:
 *         the best k moves with the device and the matrix shape): it preprocesses with
 *         k = 4, 6, 8, 10, 12 (4..8 for RSR_TERNARY_FUSED), times the multiply kernel of
 *         each on this device with both vector types and keeps the fastest;
 *         rsr_block_height() tells the choice.  RSR_BINARY / RSR_TERNARY_2PASS: 1..15;
 *         RSR_TERNARY_FUSED: 1..10.  The vector, one float per pattern (P = 2^k or 3^k;
 *         or, when P is much larger than cols, one float per non-empty pattern of a
 *         block) and about 10 KiB must fit the 160 KiB of LDS, else RSR_EUNSUPPORTED.
 *         Ignored for RSR_DENSE_TERNARY_P2.
 *
 * Pattern code of column j in block b: row b*k+r is digit r, least
 * significant first; binary digits {0,1} base 2; fused digits 0,1,2 for
 * 0,+1,-1 base 3.  The handle keeps, per pass, the canonical artifacts
 * (column permutation pi, group boundaries off; see the getters) and the
 * compact stream the multiply kernel reads: 16-bit column entries with one tail flag per
 * group (8-bit entries, tail bits and one sign word per existing group when cols <= 256);
 * the per-group prefix array of the kernel is indexed by pattern code, or by the rank of the
 * group among the existing ones when P is much larger than cols.
 *
 * Runs on the current HIP device, on the null stream, and synchronises
 * before returning.  Returns NULL on failure (see rsr_last_error()).
 * The handle owns its device buffers until rsr_destroy().
 */
rsr_handle_t rsr_preprocess(const int8_t *M, int64_t rows, int64_t cols, int k, int kind);

/*
 * rsr_matvec -- the online phase (paper, System Overview: aggregate the
 * entries of v of each group, distribute each group sum once; Kernels
 * Implementation: gather, aggregate and scatter phases).
 *
 *   v      DEVICE pointer, float32 [cols]
 *   out    DEVICE pointer, float32 [rows]; overwritten (no accumulate)
 *   stream hipStream_t passed as void*; NULL = the null stream
 *
 * Asynchronous on `stream`; allocates nothing and never synchronises, so it
 * may be captured into a HIP graph.  The current device must be the one the
 * handle was made on (RSR_EINVAL otherwise).  Calls on different streams with
 * different `out` may overlap.  Accumulation is float32.
 */
int rsr_matvec(rsr_handle_t h, const void *v, void *out, void *stream);

/*
 * rsr_matvec_ex -- rsr_matvec with a vector type, an output scale and a batch
 * of independent vectors.
 *
 *   v_dtype RSR_F32 or RSR_BF16 (bf16 inputs are widened exactly; accumulation
 *           and output stay float32)
 *   scale   per-tensor scale applied to every output
 *   batch   number of vectors (>= 1); vector i starts at v + i*ldv elements,
 *           its result at out + i*ldo elements (ldv >= cols, ldo >= rows)
 *
 * A batch is one launch.  The dense kind multiplies up to 16 vectors per pass over the
 * weights.  The RSR kinds give every vector its own workgroups (the weight side is then
 * read from HBM once and from the caches by the other vectors).  The result of a vector
 * does not depend on the batch it is part of (bit for bit).
 */
int rsr_matvec_ex(rsr_handle_t h, const void *v, int v_dtype, float scale, void *out,
                  int batch, int64_t ldv, int64_t ldo, void *stream);

/*
 * rsr_preprocess_transposed -- the handle of the transposed matrix: the product it serves is
 * out[cols] = M^T * v[rows], i.e. the row vector v^T M that the paper's footnote on the
 * original RSR formulation multiplies.  M as for rsr_preprocess (DEVICE int8 [rows][cols]);
 * here rows <= 32766 (they become the inputs).  Transposes on the GPU, then preprocesses.
 */
rsr_handle_t rsr_preprocess_transposed(const int8_t *M, int64_t rows, int64_t cols, int k, int kind);

/*
 * rsr_preprocess_stacked / rsr_matvec_stacked -- sibling layers that share their input
 * (paper, Kernels Implementation: the Q, K and V projections, and gate and up, are batched
 * into one operation over a larger pool of row blocks).  One handle over n matrices with
 * the same `cols`; one launch multiplies them all by the same v, every layer with its own
 * scale and its own output vector.  No block mixes rows of two layers (each layer is
 * completed with zero rows to whole blocks), so per layer the canonical artifacts are those
 * of rsr_preprocess of that layer, block for block: rsr_get_perm / rsr_get_offsets return
 * the layers' blocks one layer after the other.
 *
 *   Ms      HOST array of n DEVICE pointers; Ms[i] is int8 row-major [rows[i]][cols], borrowed
 *   rows    HOST array of the n row counts (>= 1 each); n <= 8 (RSR_EUNSUPPORTED beyond)
 *   k, kind as for rsr_preprocess (k = 0: chosen by timing the stacked handle)
 *   scales  HOST array of n per-layer scales, or NULL for all ones
 *   outs    HOST array of n DEVICE float32 pointers, outs[i] of length rows[i]; overwritten
 *
 * rsr_matvec_stacked is asynchronous on `stream`, allocates nothing (the pointers and
 * scales travel as kernel arguments) and takes one vector.  rsr_matvec / rsr_matvec_ex,
 * rsr_serialize and rsr_preprocess_into refuse a stacked handle.
 */
rsr_handle_t rsr_preprocess_stacked(const int8_t *const *Ms, const int64_t *rows, int n, int64_t cols,
                                    int k, int kind);
int rsr_matvec_stacked(rsr_handle_t h, const void *v, int v_dtype, const float *scales,
                       void *const *outs, void *stream);
int rsr_num_layers(rsr_handle_t h);       /* layers of a stacked handle; 0 otherwise */

/*
 * Artifact reuse (paper, System Overview: the matrices are fixed, preprocessing is one-time
 * and its result is kept): a handle as a flat byte string and back.
 *
 *   rsr_serialized_size  bytes rsr_serialize writes for h (-1 on a bad handle)
 *   rsr_serialize        copies the handle to the HOST buffer host_buf of `capacity` bytes
 *                        (RSR_EINVAL when too small); synchronous
 *   rsr_deserialize      a new handle on the current device from `size` HOST bytes written by
 *                        rsr_serialize of this library version.  The header is checked against
 *                        every limit rsr_preprocess enforces and against the sizes it implies
 *                        (RSR_EINVAL otherwise); the stream contents are taken as they are, so
 *                        a damaged stream yields wrong products, never an out-of-range access
 *                        to device memory (stream entries only ever address LDS).
 */
int64_t rsr_serialized_size(rsr_handle_t h);
int rsr_serialize(rsr_handle_t h, void *host_buf, int64_t capacity);
rsr_handle_t rsr_deserialize(const void *host_buf, int64_t size);

/*
 * rsr_preprocess_into -- rsr_preprocess for callers that cannot allocate device memory
 * (serving loops that must not call hipMalloc, harnesses that forbid it, code that runs
 * next to a HIP graph capture): preprocesses a new matrix of the SAME shape into the
 * buffers of an existing handle, replacing the matrix it held.  Block height, kind and
 * the multiply-kernel layout stay those of the handle.  Calls no hipMalloc / hipFree and
 * no allocating library routine; the same kernels as rsr_preprocess run, and their
 * temporaries (pattern codes, the stream in logical order, per-block lengths, flags)
 * live in one fixed device array of RSR_INTO_SCRATCH_BYTES that the library holds on
 * every GPU it runs on until the process ends.
 *
 *   h  a handle made by rsr_preprocess / rsr_deserialize on the current device
 *   M  DEVICE int8 [rows][cols] with the handle's rows and cols; borrowed
 *
 * Temporary memory needed: 256 bytes for the dense kind; otherwise, each term rounded
 * up to 256 bytes, 256 + 2*nb*cols (pattern codes) + 1024*nb*S (the stream in logical
 * order; not for matrices of at most 256 columns, whose layout is written directly)
 * + 2*nb*slots (group codes; only for handles whose prefix array is indexed by group rank),
 * with nb = ceil(rows/k), S the 512-entry slabs per block and slots the prefix-array
 * length of the handle.  More than
 * RSR_INTO_SCRATCH_BYTES: RSR_ESCRATCH, handle untouched.  A matrix whose stream needs
 * more slots per block than the handle holds (more empty pattern groups than the matrix
 * the handle was made from): RSR_EUNSUPPORTED; an entry outside the alphabet: RSR_EVALUE.
 * After these two, and after RSR_EHIP, the handle's contents are unspecified and
 * rsr_matvec refuses it (RSR_EINVAL) until a later rsr_preprocess_into succeeds.
 *
 * Runs on the null stream and synchronises before returning.  All calls on one GPU share
 * the one scratch array: calls that overlap on a GPU (from several threads) race, and so
 * does a multiply on the same handle that overlaps the call.
 */
#define RSR_INTO_SCRATCH_BYTES (32 * 1024 * 1024)
int rsr_preprocess_into(rsr_handle_t h, const int8_t *M);

/* Frees the handle and its device buffers.  NULL is allowed. */
void rsr_destroy(rsr_handle_t h);

/* Code of the last failure on the calling thread, and a static description. */
int rsr_last_error(void);
const char *rsr_error_string(int code);

/*
 * Inspection (for parity checks and for the benchmark's byte model).
 * `pass` is 0 for one-pass kinds; for RSR_TERNARY_2PASS pass 0 is M+ and
 * pass 1 is M-.  Host buffers are caller-allocated.
 *
 *   rsr_get_perm     HOST uint32 [nb][cols]: pi of every block -- columns in
 *                    ascending pattern code, ascending column inside a group
 *   rsr_get_offsets  HOST uint32 [nb][P+1]: group c of block b is
 *                    pi[b][off[b][c] .. off[b][c+1])
 *   rsr_get_packed   HOST uint8 [rows][ceil(cols/4)] (dense kind only): entry j
 *                    in bits 2*(j%4).. of byte j/4; 00 = 0, 01 = +1, 11 = -1
 * Not valid for the other family of kinds: RSR_EINVAL.
 */
int rsr_get_perm(rsr_handle_t h, int pass, uint32_t *host_pi);
int rsr_get_offsets(rsr_handle_t h, int pass, uint32_t *host_off);
int rsr_get_packed(rsr_handle_t h, uint8_t *host_packed);

int64_t rsr_num_blocks(rsr_handle_t h);   /* nb = ceil(rows/k); 0 for the dense kind */
int rsr_block_height(rsr_handle_t h);     /* k of the handle; 0 for the dense kind    */
int64_t rsr_num_patterns(rsr_handle_t h); /* P per pass; 0 for the dense kind        */
int rsr_num_passes(rsr_handle_t h);       /* 1 or 2; 0 for the dense kind            */

/*
 * Bytes one call of rsr_matvec_ex must move between HBM and the chip with
 * this handle's layout: every weight-side byte the kernel reads once, plus
 * batch * (cols * sizeof(v element) + rows * 4).  -1 on a bad argument.
 */
int64_t rsr_algorithmic_bytes(rsr_handle_t h, int v_dtype, int batch);

/*
 * Measurement aids (the benchmark's reference legs; no part of the method).
 *
 *   rsr_launch_shape  launch geometry of the multiply kernel of an RSR handle for a vector
 *                     type: workgroups per vector, threads per workgroup, LDS bytes per
 *                     workgroup (any of the three pointers may be NULL)
 *   rsr_probe_empty   launches a kernel that does nothing with the given geometry: what a
 *                     launch costs in a sequence before it moves a byte
 *   rsr_probe_read    launches a kernel that reads `bytes` (a multiple of 1024, DEVICE
 *                     memory at src) once, 1 KiB per wave and request, every wave a
 *                     contiguous share, all requests of a wave up front -- the access
 *                     pattern of the multiply kernel's stream -- and discards the data;
 *                     `sink` is a DEVICE word that is never written in practice (may be NULL)
 * Asynchronous on `stream`, no allocation.
 */
int rsr_launch_shape(rsr_handle_t h, int v_dtype, int *workgroups, int *threads, int *lds_bytes);
int rsr_probe_empty(int workgroups, int threads, int lds_bytes, void *stream);
int rsr_probe_read(const void *src, int64_t bytes, int workgroups, int threads, void *sink, void *stream);

/*
 * Name of the multiply kernel this handle launches for a vector type (the
 * symbol a profiler reports; the same for every batch size), or NULL on a bad
 * argument.  Static storage (per thread; the next call overwrites it).
 */
const char *rsr_kernel_name(rsr_handle_t h, int v_dtype);

#ifdef __cplusplus
}
#endif
#endif /* RSR_H */
