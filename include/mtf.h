/*
 * mtf.h — C ABI of the per-processor lowered-einsum path of a mesh-laid-out Transformer layer
 * (Mesh-TensorFlow, arXiv 1811.02084) for AMD MI355X (gfx950).
 *
 * The paper states the problem as: tensors with NAMED dimensions, an n-dimensional MESH of
 * processors with named dimensions, a global COMPUTATION LAYOUT (partial map tensor-dim ->
 * mesh-dim) and, for one processor, its COORDINATE in the mesh.  From these follow the slice
 * of every tensor that processor holds and the local einsum it runs; an einsum whose
 * reduced-out dimension is split leaves a PARTIAL SUM that an Allreduce over the matching
 * mesh dimensions completes.  This library computes exactly one processor's share.
 *
 * Conventions (all entry points)
 *   - Return value: MTF_OK (0) or a negative mtf_status.  Nothing throws or aborts across the
 *     ABI.  Arguments are validated before anything is written or launched, so every error
 *     except MTF_ERR_HIP leaves all outputs untouched; MTF_ERR_HIP (a failed launch in the
 *     middle of a multi-kernel step) may leave device outputs partly written.
 *     mtf_last_error() gives a thread-local text.
 *   - Tensors are dense, row-major in the order their dims are listed, 16-byte aligned.
 *   - "host" pointers are ordinary memory; "device" pointers are HIP device memory owned by
 *     the caller.  The library never allocates or frees device memory; scratch comes in
 *     through `workspace` arguments sized by the mtf_*_workspace_bytes() calls.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Device calls
 *     are asynchronous on it; the library never synchronises.
 *   - Host-only calls (mtf_slice, mtf_einsum_plan, mtf_einsum_local_path, mtf_reshape_plan,
 *     rank/coord helpers, *_workspace_bytes, mtf_status_string) touch no GPU and work on a
 *     machine without one.
 *
 * Contents: slices and lowering plans (host); slice gather, the local einsum with its fused
 * epilogues (also cut into ranges of its contracted dim), partial-sum reduce (the Allreduce stand-in on a virtual mesh; also with a
 * component-wise epilogue), the data-parallel
 * training step; component-wise
 * addition with implicit broadcasting, local reductions; reshape on a virtual mesh (renaming,
 * and changing rank or sizes); layer normalisation over d_model; the vocabulary-split operations;
 * fixed steps of the model-parallel Transformer layer (feed-forward with and without bias,
 * attention core at head widths 128 and 256, multi-head attention, whole layer); measurement aids.
 */
#ifndef MTF_H_
#define MTF_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MTF_MAX_RANK 8 /* dims per tensor and per mesh */

/* A named dimension (section "Mesh-TensorFlow: Beyond Batch Splitting": tensor dims and mesh
 * dims both carry names; the code fragment of the worked example builds them as (name, size)). */
typedef struct {
  const char* name; /* host, NUL-terminated, owned by caller */
  int64_t size;     /* > 0 */
} mtf_dim;

/* Ordered list of named dims: a tensor shape (row-major, first dim slowest) or a mesh shape. */
typedef struct {
  const mtf_dim* dims; /* host */
  int32_t rank;        /* 0..MTF_MAX_RANK */
} mtf_shape;

/* One pair of the computation layout: tensor dim `tensor_dim` is split over mesh dim `mesh_dim`. */
typedef struct {
  const char* tensor_dim;
  const char* mesh_dim;
} mtf_rule;

/* Where the computation runs: mesh shape, global computation layout, this processor's
 * coordinate (one entry per mesh dim, host array of length mesh.rank). */
typedef struct {
  mtf_shape mesh;
  const mtf_rule* rules; /* host, may be NULL when n_rules == 0 (everything replicated) */
  int32_t n_rules;
  const int64_t* coord;  /* host */
} mtf_place;

typedef enum { MTF_F32 = 0, MTF_BF16 = 1 } mtf_dtype;

/* Component-wise operation fused into the einsum's store (section "Operation Implementation",
 * component-wise paragraph: same shape and layout in and out, purely local). */
typedef enum {
  MTF_EPI_NONE = 0,
  MTF_EPI_RELU = 1,     /* out = max(value, 0) */
  MTF_EPI_MASK_GT0 = 2, /* out = aux > 0 ? value : 0; aux has out's shape and the input dtype */
  /* The worked example's hidden layer, h = Relu(einsum(x, w) + bias): aux is a tensor over the
   * output's innermost dim (input dtype), implicitly broadcast over the other dims (section
   * "Mesh-TensorFlow syntax": binary component-wise operations broadcast an operand whose
   * shape is a subset of the other's). */
  MTF_EPI_BIAS = 3,      /* out = value + aux[innermost index] */
  MTF_EPI_BIAS_RELU = 4  /* out = max(value + aux[innermost index], 0) */
} mtf_epilogue;

typedef enum { MTF_REDUCE_SUM = 0, MTF_REDUCE_MAX = 1 } mtf_reduce_op;

typedef enum {
  MTF_OK = 0,
  MTF_ERR_NULL = -1,             /* required pointer is NULL */
  MTF_ERR_DUP_DIM = -2,          /* two identically named dims in one tensor / mesh / output */
  MTF_ERR_SIZE_MISMATCH = -3,    /* one name, different sizes across operands; size <= 0 */
  MTF_ERR_INDIVISIBLE = -4,      /* split dim not divisible by the mesh dim's size */
  MTF_ERR_LAYOUT_CONFLICT = -5,  /* two dims of one tensor (or of one einsum) on one mesh dim */
  MTF_ERR_DUP_RULE = -6,         /* a tensor dim appears in two layout rules */
  MTF_ERR_UNKNOWN_MESH_DIM = -7, /* a rule names a mesh dim the mesh lacks */
  MTF_ERR_COORD_RANGE = -8,      /* coordinate / rank outside the mesh */
  MTF_ERR_OUT_NOT_SUBSET = -9,   /* output dim present in no input */
  MTF_ERR_UNSUPPORTED = -10,     /* legal request this build has no kernel for */
  MTF_ERR_WORKSPACE = -11,       /* workspace missing or too small */
  MTF_ERR_HIP = -12,             /* a HIP runtime call failed (text in mtf_last_error) */
  MTF_ERR_RANK = -13,            /* rank outside 0..MTF_MAX_RANK */
  MTF_ERR_ALIGN = -14            /* device pointer not 16-byte aligned */
} mtf_status;

const char* mtf_status_string(int code);
const char* mtf_last_error(void); /* thread-local; valid until the thread's next failing call */

/* ---------------------------------------------------------------- host: mesh numbering
 * Processors are numbered row-major over the mesh shape, last mesh dim fastest; this is what
 * lets one set of processors be viewed as meshes [16,16,2], [32,16] or [512] (section
 * "Hardware Assumptions").  coord: host array, length mesh->rank. */
int mtf_rank_to_coord(const mtf_shape* mesh, int64_t rank, int64_t* coord);
int mtf_coord_to_rank(const mtf_shape* mesh, const int64_t* coord, int64_t* rank);

/* ---------------------------------------------------------------- host: slice of a tensor
 * Section "Tensor Representations".  The tensor's layout is the restriction of the computation
 * layout to its dims (rules naming other dims are ignored) and must be injective.  A dim mapped
 * to mesh dim m of size n_m keeps the contiguous stripe [c*size/n_m, (c+1)*size/n_m) for
 * coordinate c; other dims are kept whole.  offset/size: host arrays of length t->rank.
 * Errors: NULL, RANK, DUP_DIM, SIZE_MISMATCH, DUP_RULE, UNKNOWN_MESH_DIM, COORD_RANGE,
 * LAYOUT_CONFLICT, INDIVISIBLE. */
int mtf_slice(const mtf_shape* t, const mtf_place* p, int64_t* offset, int64_t* size);

/* ---------------------------------------------------------------- host: lowering of one einsum
 * Section "Operation Implementation", einsum paragraph: the einsum runs locally on the slices;
 * the result must then be summed over every mesh dim that a reduced-out, split tensor dim maps
 * to.  a, b, out are GLOBAL shapes (b may be NULL for a one-operand einsum).  Outputs (any may
 * be NULL): local sizes of a, b, out (host arrays of the operand's rank); bit m of
 * *reduce_mesh_dims_mask set iff the partial result needs an Allreduce over mesh dim m;
 * *flops_local = 2 x local iteration-space size (Appendix B, "Iteration Space").
 * The union of the operands' dims obeys the same injectivity rule as a single tensor.
 * Additional errors: OUT_NOT_SUBSET. */
int mtf_einsum_plan(const mtf_shape* a, const mtf_shape* b, const mtf_shape* out,
                    const mtf_place* p, int64_t* a_local, int64_t* b_local, int64_t* out_local,
                    uint32_t* reduce_mesh_dims_mask, int64_t* flops_local);

/* ---------------------------------------------------------------- device: slice gather / scatter
 * Copies the slice mtf_slice() describes between a full tensor and a contiguous slice buffer
 * (scatter = 0: slice <- full, `full` is only read;  scatter != 0: full <- slice, `slice` is only
 * read).  full, slice: device.  Bit-exact. */
int mtf_slice_copy(void* full, void* slice, const mtf_shape* t, const mtf_place* p,
                   mtf_dtype dt, int scatter, void* stream);

/* ---------------------------------------------------------------- device: the local einsum
 * out[out dims] (+)= alpha * sum over dims not in out of a[...] * b[...], then the epilogue.
 * Shapes are LOCAL (what mtf_einsum_plan returned); names decide everything (einsum paragraph
 * of "Operation Implementation").  in_dt is the dtype of a, b and aux; accumulation is fp32.
 * accumulate != 0 adds to the existing out (read in out_dt) before the epilogue.
 * bf16 operands whose dims fold to a (batched) matrix product run on MFMA; a one-operand einsum
 * that keeps every dim in place (a component-wise operation: scale, ReLU, mask) runs as a
 * vectorised pass; anything else runs on a generic fp32 FMA kernel.  b may be NULL (one-operand
 * einsum: component-wise operations, reductions, transposes).
 * Errors: NULL, RANK, DUP_DIM, SIZE_MISMATCH, OUT_NOT_SUBSET, ALIGN, UNSUPPORTED, HIP. */
int mtf_einsum_local(const void* a, const mtf_shape* a_local, const void* b,
                     const mtf_shape* b_local, void* out, const mtf_shape* out_local,
                     mtf_dtype in_dt, mtf_dtype out_dt, mtf_epilogue epi, const void* aux,
                     float alpha, int accumulate, void* stream);

/* The same einsum with its contracted dim cut into n (1..4) equal ranges, as one launch:
 * outs[i] (fp32, each of the output's local shape) receives the sum over range i, and their sum
 * is the einsum.  For einsums whose output is too narrow to give every CU a tile and whose
 * result is a partial sum on its way into mtf_reduce_partials anyway (a contracted, split dim;
 * einsum paragraph of "Operation Implementation"): the reduce then simply takes n times as many
 * buffers - on one GPU the same thing the layout does across processors when it splits a
 * reduced-out dim.  bf16 operands that fold to one matrix product without batch dims only
 * (mtf_einsum_local_path says MTF_PATH_MFMA for them) and a contracted size divisible by 8 n;
 * anything else is MTF_ERR_UNSUPPORTED and nothing is launched.  outs: HOST array of n DEVICE
 * pointers.  Errors: as mtf_einsum_local. */
int mtf_einsum_local_kranges(const void* a, const mtf_shape* a_local, const void* b,
                             const mtf_shape* b_local, void* const* outs, int32_t n,
                             const mtf_shape* out_local, void* stream);

/* Which kernel mtf_einsum_local would run for exactly these arguments: MTF_PATH_MFMA (the bf16
 * matrix-core kernel) or MTF_PATH_GENERIC (one thread per output element, fp32 FMA: the same
 * result up to summation order, one to two orders of magnitude slower at layer sizes), or the
 * negative status mtf_einsum_local would return.  The generic kernel takes over for fp32 inputs,
 * one-operand einsums, dim structures that do not fold to a (batched) matrix product, extents or
 * leading dims not divisible by 8 (odd leading dims), leading dims too large for the kernel's
 * 32-bit offsets, and a bias over an output dim that was merged with its neighbour.  Host only:
 * looks at shapes and addresses, launches nothing, needs no GPU. */
#define MTF_PATH_GENERIC 0
#define MTF_PATH_MFMA 1
#define MTF_PATH_COMPONENTWISE 2 /* one operand, every dim kept in place: a vectorised HBM-bound pass */
int mtf_einsum_local_path(const void* a, const mtf_shape* a_local, const void* b,
                          const mtf_shape* b_local, void* out, const mtf_shape* out_local,
                          mtf_dtype in_dt, mtf_dtype out_dt, mtf_epilogue epi, const void* aux,
                          float alpha, int accumulate);

/* ---------------------------------------------------------------- device: partial-sum reduce
 * out[i] = (residual ? residual[i] : 0) + partials[0][i] + ... + partials[n-1][i], summed in
 * fp32 in that fixed order.  Stands in, on one GPU, for the Allreduce over one group of a
 * virtual mesh (the per-column sums of the 2-D layout of the worked example, section
 * "Data-Parallel, Model-Parallel Layouts").
 * partials: HOST array of n (1..64) DEVICE pointers to fp32 buffers of `count` elements. */
int mtf_reduce_partials(const void* const* partials, int32_t n, const void* residual,
                        mtf_dtype residual_dt, void* out, mtf_dtype out_dt, int64_t count,
                        void* stream);
/* The same with a component-wise operation on the complete sum (section "Operation
 * Implementation", component-wise paragraph: no communication, so it can ride on the pass that
 * ends the Allreduce): MTF_EPI_RELU: out = max(sum, 0); MTF_EPI_MASK_GT0: out = aux > 0 ?
 * sum : 0 with aux a DEVICE bf16 buffer of `count` elements (the saved activation: the ReLU
 * gradient).  In the layouts that split d_model the pre-activation is itself a partial sum, so
 * the ReLU can only follow the reduce; this is that pair in one pass.  Bit-identical to
 * mtf_reduce_partials followed by the component-wise mtf_einsum_local.
 * Errors: as mtf_reduce_partials; UNSUPPORTED for any other epilogue; NULL / ALIGN for aux. */
int mtf_reduce_partials_epi(const void* const* partials, int32_t n, const void* residual,
                            mtf_dtype residual_dt, void* out, mtf_dtype out_dt, int64_t count,
                            mtf_epilogue epi, const void* aux, void* stream);

/* ---------------------------------------------------------------- device: the data-parallel training step
 * Section "Inspiration: Single-Program-Multiple-Data (SPMD) Batch-Splitting", Algorithm 1, steps
 * 2 and 3 for one parameter tensor: the gradients the n processors of the data-parallel group
 * computed on their sub-batches are summed (the Allreduce; on one GPU the sum of the virtual
 * processors' buffers, in the fixed order 0, 1, ...) and the parameter is updated.  The paper
 * leaves Update open: plain gradient descent, master <- master - lr * sum.
 * grads: HOST array of n (1..64) DEVICE pointers to fp32 buffers of `count` elements; master:
 * device fp32, in and out (the full-precision copy of the parameter); weights: device bf16, out,
 * the rounded copy the einsums read (may be NULL).  Errors: NULL, UNSUPPORTED, SIZE_MISMATCH,
 * ALIGN, HIP. */
int mtf_sgd_step(const void* const* grads, int32_t n, float lr, void* master, void* weights,
                 int64_t count, void* stream);

/* ---------------------------------------------------------------- reshape (same sizes, new names)
 * Subsection "Reshape": keeping the dim sizes and changing dim names changes the layout, and
 * with it what each processor must hold.  `in` and `out` are GLOBAL shapes of equal rank and
 * sizes.  Per mesh dim m, comm[m] (host array of mesh.rank entries) is the communication among
 * the processors that differ only along m:
 *   NONE       the same position is split over m before and after, or none is;
 *   SLICE      a position becomes split over m: slicing on each processor, no communication;
 *   ALLGATHER  a position was split over m and is not any more;
 *   ALLTOALL   different positions are split over m before and after (e.g. switching between
 *              data- and model-parallelism).
 * Errors: those of mtf_slice for either shape; SIZE_MISMATCH if rank or sizes differ. */
typedef enum { MTF_COMM_NONE = 0, MTF_COMM_SLICE = 1, MTF_COMM_ALLGATHER = 2, MTF_COMM_ALLTOALL = 3 } mtf_comm;
int mtf_reshape_plan(const mtf_shape* in, const mtf_shape* out, const mtf_place* p, int32_t* comm);

/* The reshape on a virtual mesh held on one GPU: writes the output slice of the processor at
 * p->coord, gathering from the input slices of all processors - what the collectives of
 * mtf_reshape_plan deliver to it.  in_slices: HOST array of (product of mesh sizes, at most 64)
 * DEVICE pointers, indexed by processor rank (mtf_coord_to_rank), each that processor's slice of
 * `in` (contiguous, mtf_slice's sizes).  Where several processors hold a copy of an element,
 * the one with this processor's coordinates on the uninvolved mesh dims is read.  Bit-exact. */
int mtf_reshape_virtual(const void* const* in_slices, const mtf_shape* in, const mtf_shape* out,
                        const mtf_place* p, void* out_slice, mtf_dtype dt, void* stream);

/* A reshape that changes rank or dim sizes (subsection "Reshape", first sentence: simple in the
 * non-distributed case, communication in the distributed one): the elements keep their row-major
 * order, `out` (GLOBAL shape, same number of elements as `in`, its own names) is laid out by its
 * names.  Same arguments and conventions as mtf_reshape_virtual; an element of the output slice is
 * fetched from the input slice of the processor whose coordinates are the stripes the element's
 * position in `in` falls in (this processor's own coordinates on mesh dims that split no dim of
 * `in`).  The paper names no collective for this case; on the virtual mesh it is a gather.
 * Bit-exact.  Errors: those of mtf_slice for either shape; SIZE_MISMATCH if the element counts
 * differ; RANK for a rank-0 shape; UNSUPPORTED above 64 processors. */
int mtf_reshape_general_virtual(const void* const* in_slices, const mtf_shape* in, const mtf_shape* out,
                                const mtf_place* p, void* out_slice, mtf_dtype dt, void* stream);

/* ---------------------------------------------------------------- device: component-wise addition
 * Section "Mesh-TensorFlow syntax": out = a + b where b's dims are a subset of a's (any order);
 * b is repeated along the dims it lacks.  out has a's shape.  Section "Operation
 * Implementation", component-wise paragraph: each processor applies this to its slices (LOCAL
 * shapes; the slices of a, b and out follow from one computation layout), no communication.
 * a, b are in_dt, out is out_dt; the sum is taken in fp32.
 * Errors: NULL, RANK, DUP_DIM, SIZE_MISMATCH, OUT_NOT_SUBSET (b has a dim a lacks), ALIGN, HIP. */
int mtf_add_broadcast(const void* a, const mtf_shape* a_local, const void* b,
                      const mtf_shape* b_local, void* out, mtf_dtype in_dt, mtf_dtype out_dt,
                      void* stream);

/* ---------------------------------------------------------------- device: local reduction
 * Section "Operation Implementation", paragraph "Reduction": the output dims are a subset of
 * the input dims (any order); every other dim is summed or maximised out.  This is the LOCAL
 * reduction of one slice; mtf_einsum_plan(in, NULL, out, ...) gives the local shapes and the mesh
 * dims the result must still be combined over (sum: mtf_reduce_partials).
 * Accumulation is fp32, in a fixed order (results are reproducible run to run).
 * workspace: device scratch of mtf_reduce_local_workspace_bytes() (may be 0 bytes / NULL then).
 * Errors: NULL, RANK, DUP_DIM, SIZE_MISMATCH, OUT_NOT_SUBSET, ALIGN, WORKSPACE, UNSUPPORTED, HIP. */
size_t mtf_reduce_local_workspace_bytes(const mtf_shape* in_local, const mtf_shape* out_local);
int mtf_reduce_local(const void* in, const mtf_shape* in_local, void* out,
                     const mtf_shape* out_local, mtf_dtype in_dt, mtf_dtype out_dt,
                     mtf_reduce_op op, void* workspace, size_t workspace_bytes, void* stream);

/* mtf_reduce_local for callers that cannot allocate device memory or carry a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments minus
 * the workspace, same kernels, bit-identical results.  The scratch (the chunk partials of a
 * column reduction) is a static device array inside the library, MTF_REDUCE_STATIC_MAX_SCRATCH
 * bytes per GPU, held until the process ends.  The call allocates and frees nothing and does not
 * synchronise.  A reduction whose mtf_reduce_local_workspace_bytes() exceeds the maximum is
 * rejected with MTF_ERR_WORKSPACE (nothing launched).  All calls on one GPU share that GPU's
 * array: calls that overlap in time on one GPU (different streams or host threads) race; calls
 * ordered on one stream are safe (every partial a call reads it has written itself, so nothing
 * needs clearing between calls). */
#define MTF_REDUCE_STATIC_MAX_SCRATCH (4u << 20)
int mtf_reduce_local_static(const void* in, const mtf_shape* in_local, void* out,
                            const mtf_shape* out_local, mtf_dtype in_dt, mtf_dtype out_dt,
                            mtf_reduce_op op, void* stream);

/* ---------------------------------------------------------------- device: layer normalisation
 * The paper's Transformer is the original one, where every sublayer output is normalised:
 * LayerNorm(x + Sublayer(x)).  In the paper's terms (section "Operation Implementation") that is
 * two reductions over d_model (paragraph "Reduction": the mean, then the mean squared deviation)
 * and component-wise operations with implicit broadcasting (paragraph "Component-wise
 * Operations"): y = gain * (x - mean) / sqrt(var + eps) + bias, biased variance, statistics in
 * fp32.  d_model must be unsplit (both reductions local), a multiple of 8 and at most 4096.
 * x, y, dy, dx, u: device bf16 [rows, d_model] row-major (rows = product of the other dims);
 * gain, bias: device bf16 [d_model]; mean, rstd = 1/sqrt(var + eps): device fp32 [rows], saved for
 * the backward; dgain, dbias: device fp32 [d_model].  eps >= 0.
 * Errors: NULL, SIZE_MISMATCH, UNSUPPORTED, ALIGN, WORKSPACE, HIP. */
int mtf_layer_norm_fwd(const void* x, const void* gain, const void* bias, float eps, int64_t rows,
                       int64_t d_model, void* y, void* mean, void* rstd, void* stream);

/* The same as the tail of the pass that completes a sublayer: u = residual + sum of n (1..4) fp32
 * partial sums [rows, d_model] (what the Allreduce of a one-slice group and the residual add
 * deliver; added in the order residual, partial 0, 1, ...; u stored bf16), then the
 * normalisation of the STORED u: one pass over the data instead of mtf_reduce_partials followed
 * by mtf_layer_norm_fwd, with bit-identical u, y and statistics. */
int mtf_residual_layer_norm_fwd(const void* const* partials, int32_t n, const void* residual,
                                const void* gain, const void* bias, float eps, int64_t rows,
                                int64_t d_model, void* u, void* y, void* mean, void* rstd,
                                void* stream);

/* Gradients of sum(y * dy): dx = rstd * (g - mean_d(g) - xhat * mean_d(g * xhat)) with
 * xhat = (x - mean) * rstd, g = gain * dy; dgain = sum over rows of dy * xhat, dbias = sum over
 * rows of dy (fixed summation order: reproducible run to run).  x is the tensor that was
 * normalised (u of the residual form).  workspace: device scratch of
 * mtf_layer_norm_bwd_workspace_bytes() (column partials per workgroup). */
size_t mtf_layer_norm_bwd_workspace_bytes(int64_t rows, int64_t d_model);
int mtf_layer_norm_bwd(const void* x, const void* gain, const void* mean, const void* rstd,
                       const void* dy, int64_t rows, int64_t d_model, void* dx, void* dgain,
                       void* dbias, void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------- device: vocabulary-split operations
 * Section 'Model-Parallel "Transformer"': vocab is split across the mesh like d_ff and heads.
 * The paper gives no formulas for the operations that carry vocab; they are taken as its own
 * operations: embedding = einsum(onehot(ids)[batch,length,vocab], table[vocab,d_model]) (vocab
 * reduced out: a partial sum), logits = einsum(x, w[d_model,vocab]) through mtf_einsum_local
 * (vocab kept: a slice), loss = reduce_max + log reduce_sum(exp(logits - max)) - the target's
 * logit, each reduction over the split vocab completed by an Allreduce over vocab's mesh dims
 * (max: mtf_max_partials; sums: mtf_reduce_partials).  ids / targets are GLOBAL token ids
 * (device, int32); this processor holds the vocab stripe [vocab_offset, vocab_offset +
 * vocab_local) (mtf_slice of the vocab dim).  `count` / `rows` = batch * length tokens. */

/* out_partial[t, :] = table_local[ids[t] - vocab_offset, :] where that row is local, 0 elsewhere
 * (table bf16 [vocab_local, d_model]; out_partial [count, d_model] in out_dt; d_model % 8 == 0). */
int mtf_embedding_local(const void* ids, int64_t count, const void* table_local,
                        int64_t vocab_local, int64_t d_model, int64_t vocab_offset,
                        void* out_partial, mtf_dtype out_dt, void* stream);
/* dtable_local[v, :] (fp32, every row written) = sum over t with ids[t] == vocab_offset + v of
 * de[t, :] (bf16), summed in token order. */
int mtf_embedding_grad_local(const void* ids, int64_t count, const void* de, int64_t vocab_local,
                             int64_t d_model, int64_t vocab_offset, void* dtable_local,
                             void* stream);
/* out[i] = max over the n (1..64) fp32 device buffers partials[k][i]: the Allreduce(max) of one
 * group of a virtual mesh (reduce_max over a split dim).  partials: HOST array. */
int mtf_max_partials(const void* const* partials, int32_t n, void* out, int64_t count,
                     void* stream);
/* Local statistics of the loss given the (already Allreduced) row maxima row_max[rows]:
 * sumexp[r] = sum_v exp(logits_local[r, v] - row_max[r]); picked[r] = logits_local[r, targets[r] -
 * vocab_offset] if the target is local, else 0.  logits_local fp32 [rows, vocab_local].  The local
 * row maxima themselves come from mtf_reduce_local(MTF_REDUCE_MAX). */
int mtf_xent_stats_local(const void* logits_local, int64_t rows, int64_t vocab_local,
                         const void* row_max, const void* targets, int64_t vocab_offset,
                         void* sumexp, void* picked, void* stream);
/* loss[r] = row_max[r] + log(sumexp[r]) - picked[r] (all fp32, after their Allreduces). */
int mtf_xent_loss(const void* row_max, const void* sumexp, const void* picked, void* loss,
                  int64_t rows, void* stream);
/* dlogits_local[r, v] (bf16) = (exp(logits_local[r, v] - row_max[r]) / sumexp[r]
 *                               - [vocab_offset + v == targets[r]]) * dloss[r].
 * vocab_local % 4 == 0.  dW and dx then are einsums of dlogits (mtf_einsum_local). */
int mtf_xent_grad_local(const void* logits_local, int64_t rows, int64_t vocab_local,
                        const void* row_max, const void* sumexp, const void* targets,
                        int64_t vocab_offset, const void* dloss, void* dlogits_local, void* stream);

/* Element-wise dtype conversion (fp32 <-> bf16 round-to-nearest-even, or copy). */
int mtf_cast(const void* in, mtf_dtype in_dt, void* out, mtf_dtype out_dt, int64_t count,
             void* stream);

/* ---------------------------------------------------------------- device: fixed layer steps
 * One processor's share of the two sublayers of the model-parallel Transformer (section
 * 'Model-Parallel "Transformer"': d_ff and heads are split, so W_in[d_model,d_ff], W_out[d_ff,
 * d_model], W_{q,k,v}[d_model,heads,d_k], W_o[heads,d_k,d_model] are local slices and y / dx
 * are partial sums).  All sizes are LOCAL.  Activations and weights are bf16; partial sums and
 * parameter gradients are fp32.  d_v = d_k. */
typedef struct {
  int64_t batch, length, d_model, d_ff;
} mtf_ffn_dims;

typedef struct {
  int64_t batch, length, d_model, heads, d_k;
} mtf_mha_dims;

typedef struct {
  int64_t batch, length, d_model, heads, d_k, d_ff;
} mtf_layer_dims;

/* Worked example y = Relu(x w) v without bias.
 * x[batch,length,d_model], w_in[d_model,d_ff], w_out[d_ff,d_model] (bf16, in);
 * a[batch,length,d_ff] = relu(x w_in) (bf16, out, saved for backward);
 * y_partial[batch,length,d_model] (fp32, out). */
int mtf_ffn_fwd(const mtf_ffn_dims* d, const void* x, const void* w_in, const void* w_out,
                void* a, void* y_partial, void* stream);

/* The worked example as printed, y = Relu(x w + bias) v (section "Example: Two Fully-Connected
 * Layers"): as mtf_ffn_fwd with bias[d_ff] (bf16, in) added before the ReLU. */
int mtf_ffn_bias_fwd(const mtf_ffn_dims* d, const void* x, const void* w_in, const void* bias,
                     const void* w_out, void* a, void* y_partial, void* stream);

size_t mtf_ffn_bwd_workspace_bytes(const mtf_ffn_dims* d);
/* dy[batch,length,d_model] bf16 in;  dw_in[d_model,d_ff], dw_out[d_ff,d_model],
 * dx_partial[batch,length,d_model] fp32 out.  The ReLU mask is a > 0. */
int mtf_ffn_bwd(const mtf_ffn_dims* d, const void* x, const void* a, const void* w_in,
                const void* w_out, const void* dy, void* dw_in, void* dw_out, void* dx_partial,
                void* workspace, size_t workspace_bytes, void* stream);

/* As mtf_ffn_bwd, plus dbias[d_ff] (fp32, out) = reduce_sum of dh over batch and length: like
 * the other parameter gradients it reduces out `batch` ("Data-Parallel Layout"). */
size_t mtf_ffn_bias_bwd_workspace_bytes(const mtf_ffn_dims* d);
int mtf_ffn_bias_bwd(const mtf_ffn_dims* d, const void* x, const void* a, const void* w_in,
                     const void* w_out, const void* dy, void* dw_in, void* dbias, void* dw_out,
                     void* dx_partial, void* workspace, size_t workspace_bytes, void* stream);

/* Self-attention over x (memory = x).  logits = scale * q.k over d_k; softmax over the memory
 * positions; causal != 0 hides memory positions m > l.  Outputs q,k,v,ctx [batch,length,heads,
 * d_k] bf16 and lse [batch,heads,length] fp32 are saved for backward; y_partial fp32.
 * d_k must be 128 or 256 (the head widths of the paper's experiments, which have fused attention
 * kernels); another width is MTF_ERR_UNSUPPORTED here and served by mtf_attention_fwd / _bwd. */
int mtf_mha_fwd(const mtf_mha_dims* d, const void* x, const void* w_q, const void* w_k,
                const void* w_v, const void* w_o, float scale, int causal, void* q, void* k,
                void* v, void* ctx, void* lse, void* y_partial, void* stream);

size_t mtf_mha_bwd_workspace_bytes(const mtf_mha_dims* d);
int mtf_mha_bwd(const mtf_mha_dims* d, const void* x, const void* w_q, const void* w_k,
                const void* w_v, const void* w_o, const void* q, const void* k, const void* v,
                const void* ctx, const void* lse, const void* dy, float scale, int causal,
                void* dw_q, void* dw_k, void* dw_v, void* dw_o, void* dx_partial,
                void* workspace, size_t workspace_bytes, void* stream);

/* The attention core alone, for any head width d_k = d_v divisible by 8 (the LM models of the
 * paper use 256): ctx[batch,length,heads,d_k] = einsum(softmax_m(scale * einsum(q, k -> [batch,
 * heads,length,memory])), v), lse[batch,heads,length] fp32; q, k, v, ctx, dctx, dq, dk, dv bf16
 * [batch,length,heads,d_k].  d_k = 128 and d_k = 256 run the fused kernels (no workspace forward,
 * one fp32 per (batch, head, position) backward); any other width runs the two einsums on the GEMM
 * kernel with a row-softmax kernel between them and needs length % 8 == 0 and a workspace for the
 * [batch,heads,length,length] intermediates.
 * d->d_model is not used.  Errors: NULL, SIZE_MISMATCH, UNSUPPORTED, ALIGN, WORKSPACE, HIP. */
size_t mtf_attention_fwd_workspace_bytes(const mtf_mha_dims* d);
int mtf_attention_fwd(const mtf_mha_dims* d, const void* q, const void* k, const void* v,
                      float scale, int causal, void* ctx, void* lse, void* workspace,
                      size_t workspace_bytes, void* stream);
size_t mtf_attention_bwd_workspace_bytes(const mtf_mha_dims* d);
int mtf_attention_bwd(const mtf_mha_dims* d, const void* q, const void* k, const void* v,
                      const void* ctx, const void* lse, const void* dctx, float scale, int causal,
                      void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes,
                      void* stream);

/* Whole layer for a one-slice Allreduce group: u = x + MHA(x), z = u + FFN(u); u, z bf16. */
typedef struct {
  const void *w_q, *w_k, *w_v, *w_o, *w_in, *w_out; /* device, bf16 */
} mtf_layer_weights;
typedef struct {
  void *q, *k, *v, *ctx, *lse, *u, *a; /* device; lse fp32, others bf16 */
} mtf_layer_saved;
typedef struct {
  void *dw_q, *dw_k, *dw_v, *dw_o, *dw_in, *dw_out; /* device, fp32 */
} mtf_layer_grads;

size_t mtf_layer_fwd_workspace_bytes(const mtf_layer_dims* d);
int mtf_layer_fwd(const mtf_layer_dims* d, const void* x, const mtf_layer_weights* w, float scale,
                  int causal, const mtf_layer_saved* saved, void* z, void* workspace,
                  size_t workspace_bytes, void* stream);

size_t mtf_layer_bwd_workspace_bytes(const mtf_layer_dims* d);
int mtf_layer_bwd(const mtf_layer_dims* d, const void* x, const mtf_layer_weights* w,
                  const mtf_layer_saved* saved, const void* dz, float scale, int causal,
                  const mtf_layer_grads* g, void* dx, void* workspace, size_t workspace_bytes,
                  void* stream);

/* ---------------------------------------------------------------- measurement aid
 * While enabled, every kernel launch of the library is bracketed by two HIP events recorded on
 * the launch's own stream.  mtf_timing_collect() waits for those events (it synchronises with the
 * work that was timed), adds them up per kernel and forgets them.  For callers that must report
 * per-kernel time measured inside their own timed region (the benchmark); leave it off otherwise.
 * flops / bytes are the algorithmic work of the timed launches: 2 x iteration-space size for a
 * contraction (Appendix B), bytes of inputs + outputs for the HBM-bound helpers. */
typedef struct {
  char kernel[96];   /* kernel name as a profiler prints it, NUL-terminated */
  int64_t launches;
  double total_ms;
  double flops;
  double bytes;
} mtf_kernel_time;

int mtf_timing_enable(int on);
/* out: host array of max_kinds entries; *n_kinds receives the number filled. */
int mtf_timing_collect(mtf_kernel_time* out, int32_t max_kinds, int32_t* n_kinds);

/* What the matrix cores alone sustain on this device, for the roofline a contraction is held
 * against: one launch of a kernel that does nothing but v_mfma_f32_32x32x16_bf16 (8 independent
 * accumulators per wavefront, 8 wavefronts per CU on every CU), operands taken from `operands`
 * (device, bf16, at least 4096 elements; power draw, hence the sustained clock, depends on the
 * operand bits: pass values distributed like the real operands).  `iters` MFMAs per accumulator
 * (> 0).  `sink` (device, at least 66 floats): sink[0..63] receive a value derived from the
 * accumulators so the loop is not optimised away; sink[64] and sink[65] the span of the first
 * wavefront's loop in shader-clock cycles and in ticks of the constant 100 MHz clock (their ratio
 * x 100 MHz is the clock the matrix cores were running at).  *flops receives the FLOP of the
 * launch (host).  Time it with events or with mtf_timing_*: kernel name "mfma_ceiling_kernel". */
int mtf_mfma_ceiling(const void* operands, int32_t iters, void* sink, double* flops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MTF_H_ */
