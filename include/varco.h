/*
 * varco.h - C ABI of the MI355X (gfx950) library for the hot path of VARCO: one partition's step of a
 * partitioned GNN layer, forward and backward, with compressed exchange of boundary activations.
 *
 * Paper passages the calls follow
 *   eq. (1)-(2), Section II      X_l = rho( sum_k S^k X_{l-1} H_{l,k} ): aggregation, transform, nonlinearity
 *   Section III, Algorithm 1     each worker owns a node subset; per layer the owners compress the
 *                                activations of their boundary nodes, consumers decompress them and run
 *                                the forward pass on uncompressed local + compressed remote rows; errors
 *                                flow back through the same compression; weight gradients are summed
 *   Definition 1, Appendix A     compression keeps n/r elements chosen at random with a key shared
 *                                beforehand; the decoder writes them in place and zeros the rest
 *   Section IV, Appendix A       the ratio is set per training step by a decreasing scheduler
 *
 * Conventions
 *   - Every function returns a status code (VARCO_OK = 0); nothing throws or aborts. varco_last_error()
 *     gives the text of the last failure on that context (or of the last failed varco_create /
 *     varco_partition_build when ctx is NULL).
 *   - "device" pointers are HIP device memory owned by the caller; the library borrows them while the
 *     enqueued work runs and never frees them. "host" pointers are ordinary host memory.
 *   - All device work is enqueued on the caller's stream (a hipStream_t passed as void*; NULL is the
 *     default stream). Device memory is allocated, and the device possibly synchronised, only by the set-up
 *     calls: varco_register_partition, varco_prepare, varco_set_ratio (when a larger k needs a larger
 *     workspace), varco_step_table_enable (first call) and, while it is enabled, the per-kernel profiler
 *     (events). The compute calls (compress, decompress, layer, aggregate, transform, accumulate, loss, update)
 *     allocate nothing, never synchronise, and may be captured into a HIP graph.
 *   - Matrices are row-major and dense (leading dimension = width) unless a leading dimension is given.
 *   - Node ids, row ids and counts are int32 (graphs below 2^31 nodes / entries per partition); element
 *     offsets are 64-bit inside the library.
 *   - A context is not thread-safe (one host thread issues its calls). Layer calls may be issued on up
 *     to 8 different streams, whose work then may overlap on the device: the library keeps one workspace
 *     set per stream, made by varco_prepare(ctx, stream). The caller
 *     orders dependent work across streams (events), and gives calls that may overlap different output
 *     buffers; dh1 / dh0 in particular are read-modify-written (see varco_sum_gradients).
 *   - Layers are numbered 0..L-1; layer l maps width[l] -> width[l+1]. k_l is the number of elements of a
 *     width[l] vector that is communicated at the current ratio of layer l.
 */
#ifndef VARCO_H
#define VARCO_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct varco_ctx varco_ctx;
typedef struct varco_host_parts varco_host_parts;
typedef void* varco_stream;

enum {
    VARCO_OK = 0,
    VARCO_ERR_INVALID_ARG = 1, /* null pointer, index out of range, ratio < 1 */
    VARCO_ERR_SHAPE = 2,       /* sizes that do not fit together or exceed the supported range */
    VARCO_ERR_STATE = 3,       /* call order violated (unregistered partition, ratio change mid-step) */
    VARCO_ERR_UNSUPPORTED = 4, /* dtype / conv / width the kernels do not implement */
    VARCO_ERR_HIP = 5          /* a HIP runtime call failed; text in varco_last_error */
};

enum { VARCO_CONV_GCN = 0 /* single tap S */, VARCO_CONV_SAGE = 1 /* taps I (H0) and S (H1) */ };
enum { VARCO_ACT_IDENTITY = 0, VARCO_ACT_RELU = 1 };
/* Order of the two products of eq. (2) inside a layer call; see varco_set_layer_order. */
enum { VARCO_ORDER_AGGREGATE_FIRST = 0 /* (S X) H */, VARCO_ORDER_TRANSFORM_FIRST = 1 /* S (X H) */ };
enum { VARCO_F32 = 0, VARCO_BF16 = 1 /* activations and gradients stored as bf16, arithmetic in fp32 */ };

#define VARCO_MAX_LAYERS 16
#define VARCO_MAX_WIDTH 2048

/* Network description (eq. (2); Section V uses 3 layers, 256 hidden units, ReLU). Host pointers, copied. */
typedef struct {
    int32_t n_layers;       /* L, 1..VARCO_MAX_LAYERS */
    int32_t n_partitions;   /* Q of Section III */
    int32_t conv;           /* VARCO_CONV_* */
    int32_t dtype;          /* VARCO_F32 or VARCO_BF16: storage type of x, z, m_saved, dx, dz_halo; weights are fp32 */
    uint64_t mask_key;      /* the key shared a priori between encoder and decoder (Appendix A) */
    const int32_t* widths;  /* L+1 widths F_0..F_L, each 1..VARCO_MAX_WIDTH; above 512 only multiples of 4, and the
                             * activation / gradient buffers of such a width must be 16-byte aligned (else
                             * VARCO_ERR_UNSUPPORTED from create or from the layer call) */
    const int32_t* act;     /* L activation codes VARCO_ACT_* */
} varco_config;

/*
 * One partition's index structures (Section III: local nodes, remote neighbours, boundary nodes).
 * Used twice: varco_partition_view fills it with HOST pointers owned by the varco_host_parts handle;
 * varco_register_partition reads it with DEVICE pointers owned by the caller, which must stay valid and
 * unchanged until the context is destroyed or the partition is registered again.
 *
 *   row block   rowptr[n_local+1], colidx[nnz], vals[nnz]: CSR of S restricted to the partition's rows;
 *               column c < n_local is local row c, column n_local+s is halo slot s; ascending in a row
 *   transpose   t_rowptr[n_local+n_halo+1], t_colidx[nnz], t_vals[nnz]: row c lists local rows i with
 *               S[i,c] != 0, ascending
 *   local_gid[n_local] ascending global ids; halo_gid[n_halo] ordered by (owner, global id)
 *   halo_owner_ptr[n_partitions+1]: slots of owner p are [halo_owner_ptr[p], halo_owner_ptr[p+1])
 *   boundary_rows[n_boundary]: ascending local rows referenced by some other partition
 *   halo_src_row[n_halo]: position of the halo node in its owner's boundary_rows
 *   halo_zrow[n_halo]: halo_src_row + (boundary rows of all partitions before the owner) = row in the
 *               concatenated compressed buffer; z_row_offset: first row of this partition's own slice
 *   owner side of the backward exchange (Section III: errors travel from consumers back to owners). The
 *   rows returned by all consumers form one array, partition q's n_halo rows starting at row
 *   halo_row_offset = sum of n_halo over the partitions before q. For boundary row b of this partition,
 *   ret_src[ret_ptr[b] .. ret_ptr[b+1]) are the rows of that array that belong to b's node, one per consumer,
 *   consumers ascending; ret_ptr[n_boundary + 1], ret_src[n_returned], n_returned = ret_ptr[n_boundary].
 *   ret_ptr / ret_src may be NULL at registration (n_returned = 0) for callers that pass their own map to
 *   varco_accumulate_returned or use varco_decompress(accumulate = 1) per consumer.
 */
typedef struct {
    int32_t n_local, n_halo, n_boundary, z_row_offset;
    int64_t nnz;
    int32_t halo_row_offset, n_returned;
    const int32_t* rowptr;
    const int32_t* colidx;
    const float* vals;
    const int32_t* t_rowptr;
    const int32_t* t_colidx;
    const float* t_vals;
    const int32_t* local_gid;
    const int32_t* halo_gid;
    const int32_t* halo_owner_ptr;
    const int32_t* boundary_rows;
    const int32_t* halo_src_row;
    const int32_t* halo_zrow;
    const int32_t* ret_ptr;
    const int32_t* ret_src;
} varco_partition_desc;

/* Compressed elements handed off between partitions since creation (or the last reset): the quantity
 * Section V-B plots accuracy against. full_* is what ratio 1 would have moved on the same calls. */
typedef struct {
    int64_t fwd_elems[VARCO_MAX_LAYERS], bwd_elems[VARCO_MAX_LAYERS];
    int64_t full_fwd_elems[VARCO_MAX_LAYERS], full_bwd_elems[VARCO_MAX_LAYERS];
    int32_t bytes_per_elem;
} varco_stats;

/* ------------------------------------------------------------------------------------------------
 * Host-side partition builder (Section III; Appendix B: any node->partition map is accepted).
 * All pointers are host memory. rowptr[n+1] int64, colidx/vals[rowptr[n]] with ascending columns in a
 * row, part[n] in [0, n_parts). The result is owned by *out until varco_partition_free.
 * Errors: INVALID_ARG (null, part out of range, unsorted row), SHAPE (a partition with >= 2^31 entries, or
 * 2^31 or more halo rows over all partitions).
 */
int32_t varco_partition_build(int32_t n, const int64_t* rowptr, const int32_t* colidx, const float* vals,
                              const int32_t* part, int32_t n_parts, varco_host_parts** out);
int32_t varco_partition_view(const varco_host_parts* h, int32_t q, varco_partition_desc* out);
void varco_partition_free(varco_host_parts* h);

/* ------------------------------------------------------------------------------------------------
 * Context. varco_create copies cfg, sets every layer's ratio to 1 and the step to 0 (host only).
 * varco_register_partition copies the row pointers to the host once (synchronising), checks the index arrays
 * on the device (SHAPE error for columns or transposed rows out of range or not strictly ascending, a
 * transpose that does not hold the row block's entries, negative ids, a malformed boundary list or returned-row
 * map: nothing is trusted unchecked), builds the library's own work lists for that partition and keeps
 * existing workspace sets large enough; it may be called again for the same q to replace a partition.
 * varco_prepare makes (or grows) the workspace set of `stream` for the partitions registered and the ratios
 * set so far, and uploads the tables of the kept positions: call it once per stream after registration and
 * before the first compute call on that stream (a compute call on a stream without a set, or whose set a
 * later change outgrew, returns VARCO_ERR_STATE; varco_set_ratio and varco_register_partition grow existing
 * sets themselves). Host call, may synchronise the device, not capturable.
 */
int32_t varco_create(const varco_config* cfg, varco_ctx** out);
int32_t varco_destroy(varco_ctx* ctx);
int32_t varco_register_partition(varco_ctx* ctx, int32_t q, const varco_partition_desc* dev);
int32_t varco_prepare(varco_ctx* ctx, varco_stream stream);
const char* varco_last_error(const varco_ctx* ctx);

/* Algorithm 1's iteration counter t: part of the mask key, so that the kept positions are redrawn every
 * step. Also closes the previous step (ratios may change again).
 * Weights belong to a step: Algorithm 1 updates the parameters between iterations, and the library may keep
 * converted copies of the weight matrices it is given (per stream, keyed by their address) until the next
 * varco_begin_step / varco_set_step / varco_advance_step. A caller that changes a weight matrix in place calls
 * one of these before using it again; a sequence captured into a HIP graph starts with varco_advance_step. */
int32_t varco_begin_step(varco_ctx* ctx, uint64_t step);

/* Step state on the device, for callers that capture a sequence of calls in a HIP graph and replay it for
 * later steps (kernel arguments are frozen at capture, the iteration counter must not be).
 *   varco_step_table_enable  allocates (first call only: not capturable) a device copy of the step and of the
 *                            key words derived from it, fills it for the current step on `stream`; from then
 *                            on every kernel takes the key words of the kept positions from that table.
 *   varco_set_step           varco_begin_step that also refreshes the table on `stream` (works in either mode).
 *   varco_advance_step       step += 1 on the device by one small kernel on `stream` (capturable: each replay
 *                            moves on by one step), and on the host; otherwise like varco_begin_step.
 * With the table enabled varco_begin_step is a STATE error. The table is shared by all streams: work of the
 * previous step must be ordered before the call that changes the step. Host-side counters (varco_get_stats)
 * and the host's copy of the step count calls, not graph replays. */
int32_t varco_step_table_enable(varco_ctx* ctx, varco_stream stream);
int32_t varco_set_step(varco_ctx* ctx, uint64_t step, varco_stream stream);
int32_t varco_advance_step(varco_ctx* ctx, varco_stream stream);

/* How the dense products of eq. (2) (X H, and the two gradient products) are formed for fp32 storage
 * (the paper fixes no arithmetic; VARCO_BF16 contexts ignore this). terms = 3 (the default): each fp32 operand
 * is written exactly as a sum of three bf16 numbers and the six largest cross products are formed on the bf16
 * matrix units with fp32 accumulation; the dropped products are below 2^-24 of each full product, so the result
 * has the accuracy of fp32 arithmetic at well under half the cost. terms = 0: fp32 matrix instructions
 * throughout (also used, whatever the setting, for shapes the expanded form cannot take: rows not 16-byte
 * aligned). terms = 2: two terms, three products, relative error about 2^-16 per product (a faster,
 * lower-precision setting nothing in this library selects by itself). With terms 2 or 3 an operand that is
 * infinite, NaN or within 2^-9 of the fp32 overflow threshold turns the outputs it meets into NaN (fp32
 * instructions would keep an infinity times a finite number infinite); use terms = 0 where such values must
 * pass. INVALID_ARG for other values. Takes effect from the next call on. */
int32_t varco_set_matmul_terms(varco_ctx* ctx, int32_t terms);

/* Section IV / Algorithm 1 (the step that updates the compression rate): ratio r = num/den >= 1 of layer `layer`'s input
 * (-1 = every layer). k = max(1, ceil(width*den/num)); r = 1 keeps everything (lossless). den = 0 (num >= 1)
 * is the unbounded ratio, k = 0: nothing of that layer's input is exchanged, forward or backward (the
 * no-communication setting Section V compares against; on every layer: each partition works on its own
 * subgraph). With k = 0 the compressed buffers of that layer are not touched and may be NULL. STATE error if
 * the layer's positions are already in use in the current step (by compress, decompress or a forward
 * call; its backward must see the same positions). Host call: when the new k needs a larger halo-gradient
 * workspace than the prepared streams hold, it is reallocated here (synchronising the device), with a quarter
 * of head-room so that a schedule that raises k step by step reallocates rarely. */
int32_t varco_set_ratio(varco_ctx* ctx, int32_t layer, uint32_t num, uint32_t den);
/* k_l currently in force (negative status on error is not used: returns status, k through *k). */
int32_t varco_get_keep(const varco_ctx* ctx, int32_t layer, int32_t* k);

/* Definition 1, encoder: z[i, j] = x[rows[i], pi_v(j)], j < k_l, v = gids[i].
 * gids[n_rows] device; rows[n_rows] device or NULL (then row i); x device with leading dimension ldx >=
 * width[layer]; z device, n_rows x k_l dense. No index bytes are produced. */
int32_t varco_compress(varco_ctx* ctx, int32_t layer, const int32_t* gids, const int32_t* rows,
                       int64_t n_rows, const void* x, int64_t ldx, void* z, varco_stream stream);

/* Definition 1 / Appendix A, decoder. accumulate = 0: x[rows[i], :] = 0 except x[rows[i], pi_v(j)] =
 * z[i, j]. accumulate = 1: x[rows[i], pi_v(j)] += z[i, j] (the owner-side sum of returned errors); rows
 * must be distinct within one call. */
int32_t varco_decompress(varco_ctx* ctx, int32_t layer, const int32_t* gids, const int32_t* rows,
                         int64_t n_rows, const void* z, void* x, int64_t ldx, int32_t accumulate,
                         varco_stream stream);

/* Order in which varco_layer_fwd / varco_layer_bwd of `layer` form the product S X H of eq. (2). The two orders are
 * the same layer (the products associate); they differ in cost. VARCO_ORDER_AGGREGATE_FIRST (default) aggregates
 * rows of width[layer] elements - the halo rows in compressed form, k elements each - and transforms the n_local
 * sums. VARCO_ORDER_TRANSFORM_FIRST transforms every source row first - the local rows, and each halo row once from
 * its k received elements (the exchange is the same compressed one) - and aggregates rows of width[layer+1]
 * elements; the errors handed back are formed per halo row from the transposed aggregate, without a buffer of
 * per-entry products. It pays for a narrowing layer whose halo rows are referred to often or kept nearly whole
 * (k close to width[layer]); at high compression the default order moves fewer bytes.
 * Supported for bf16 storage, an identity activation, width[layer+1] <= 64 and width[layer] a multiple of 16, at most 512 (the
 * class-logit layer), else VARCO_ERR_UNSUPPORTED. A set-up call like varco_set_ratio: it may allocate and synchronise,
 * and VARCO_ERR_STATE once the layer ran forward in the current step. In this order the forward call does not
 * write m_saved (it may be NULL), and the backward call takes, as its m_saved argument, the z_in the forward call
 * was given, still holding the same rows. */
int32_t varco_set_layer_order(varco_ctx* ctx, int32_t layer, int32_t order);

/* Forward of layer `layer` on partition q (Algorithm 1's forward pass: local nodes contribute their
 * activations as they are, nodes of other partitions their compressed ones):
 *   m      = S_q [x_local ; decompress(z_in[halo_zrow])]      n_local x width[layer]
 *   x_out  = act( m h1 (+ x_local h0) )                       n_local x width[layer+1]
 *   z_out rows [z_row_offset, +n_boundary) = compress(x_out[boundary_rows]) at layer+1's k   (optional)
 * x_local: n_local x width[layer]; z_in: (all partitions' boundary rows) x k_layer, owners' slices in
 * partition order (the on-device stand-in for the exchange; may be NULL when n_halo = 0); h1, h0:
 * width[layer] x width[layer+1] (h0 NULL for GCN, required for SAGE); m_saved is written and must be kept
 * for the backward call; z_out may be NULL (must be NULL on the last layer).
 * Counts n_halo * k_layer elements as handed off forward. (A layer set to VARCO_ORDER_TRANSFORM_FIRST computes the
 * same x_out as S_q [x_local h1 ; x~_halo h1] and leaves m_saved alone: see varco_set_layer_order.) */
int32_t varco_layer_fwd(varco_ctx* ctx, int32_t layer, int32_t q, const void* x_local, const void* z_in,
                        const void* h1, const void* h0, void* x_out, void* z_out, void* m_saved,
                        varco_stream stream);

/* Backward of layer `layer` on partition q (Algorithm 1's backward pass: the gradient of the forward above,
 * taken through the compression, with the errors of remote nodes handed back to their owners):
 *   dz = dx_out * [x_out > 0] (ReLU) or dx_out;  dh1 += m_saved^T dz;  dh0 += x_local^T dz
 *   if dx_local != NULL:  dm = dz h1^T;  [dx_local ; dx_halo] = S_q^T dm;  dx_local += dz h0^T;
 *                         dz_halo[s, j] = dx_halo[s, pi_v(j)], j < k_layer, v = halo_gid[s]
 * dh1/dh0 are accumulated into (the sum over partitions is the cross-machine sum of Section III); dx_local
 * (n_local x width[layer]) and dz_halo (n_halo x k_layer) are overwritten. dx_local = NULL skips the input
 * gradient (first layer); dz_halo must then be NULL too. The owners add dz_halo with varco_decompress
 * (accumulate = 1). Counts n_halo * k_layer elements as handed off backward when dz_halo is produced. (A layer set to
 * VARCO_ORDER_TRANSFORM_FIRST produces the same results from x_local and the forward call's z_in, passed as m_saved.) */
int32_t varco_layer_bwd(varco_ctx* ctx, int32_t layer, int32_t q, const void* dx_out, const void* x_out,
                        const void* x_local, const void* m_saved, const void* h1, const void* h0, void* dh1,
                        void* dh0, void* dx_local, void* dz_halo, varco_stream stream);

/* ------------------------------------------------------------------------------------------------
 * Building blocks of the general K-tap layer of eq. (1)-(2), X_l = rho( sum_{k<K} S^k X_{l-1} H_{l,k} ): every
 * application of S (hop k = 1..K-1) has an exchange of its own, Y_k = S_q [Y_{k-1,loc} ; compressed halo rows
 * of Y_{k-1}], and the transform is a sum of dense products. varco_layer_fwd / varco_layer_bwd are these calls
 * fused for K <= 2.
 *
 * A `layer` argument of varco_compress, varco_decompress, varco_accumulate_returned and a `tap` argument below
 * may be VARCO_TAP(layer, hop): hop >= 1 selects the kept positions of that hop's exchange (hop 0 is the plain
 * layer index; each hop draws positions of its own). The ratio and k are the layer's.
 */
#define VARCO_TAP(layer, hop) ((layer) + VARCO_MAX_LAYERS * (hop))

/* One hop forward: y_out = S_q [y_local ; decompress(z_in[halo_zrow])], all n_local x width[layer]; z_in as in
 * varco_layer_fwd (compressed boundary rows of y, all owners). Counts n_halo * k elements handed off forward. */
int32_t varco_aggregate_fwd(varco_ctx* ctx, int32_t tap, int32_t q, const void* y_local, const void* z_in, void* y_out,
                            varco_stream stream);
/* One hop backward: [g_local ; c_halo] = S_q^T g_out; g_local (n_local x width[layer]) is overwritten and
 * dz_halo[s, j] = c_halo[s, pi_v(j)], j < k (n_halo x k) is what goes back to the owners (they add it with
 * varco_accumulate_returned on the same tap). Counts n_halo * k elements handed off backward. */
int32_t varco_aggregate_bwd(varco_ctx* ctx, int32_t tap, int32_t q, const void* g_out, void* g_local, void* dz_halo,
                            varco_stream stream);
/* Dense products of layer `layer` on n_rows rows (storage type for y, c, dx_out, x_out, g_out; weights fp32
 * width[layer] x width[layer+1]):
 *   varco_transform_fwd         c (+)= y h; when apply_act != 0 the layer's activation is applied to the result
 *   varco_transform_bwd_weight  dh += y^T dz,  dz = dx_out * [x_out > 0] for a ReLU layer (x_out may be NULL otherwise)
 *   varco_transform_bwd_input   g_out (+)= dz h^T
 * accumulate != 0 adds to what c / g_out hold. */
int32_t varco_transform_fwd(varco_ctx* ctx, int32_t layer, int64_t n_rows, const void* y, const void* h, void* c,
                            int32_t accumulate, int32_t apply_act, varco_stream stream);
int32_t varco_transform_bwd_weight(varco_ctx* ctx, int32_t layer, int64_t n_rows, const void* y, const void* dx_out,
                                   const void* x_out, void* dh, varco_stream stream);
int32_t varco_transform_bwd_input(varco_ctx* ctx, int32_t layer, int64_t n_rows, const void* dx_out, const void* x_out,
                                  const void* h, void* g_out, int32_t accumulate, varco_stream stream);

/* varco_transform_bwd_weight for callers that cannot allocate device memory and have no prepared stream: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc. Same arguments, same kernels,
 * same split of the reduction over the rows and therefore the same bits as varco_transform_bwd_weight on a stream
 * whose workspace holds that split; but the partial products go to a static device array of the library (32 MiB
 * per GPU, held until the process ends) instead of a workspace set, so the call needs no varco_prepare and
 * allocates nothing. VARCO_ERR_SHAPE, with the sizes in the text, when width[layer] x width[layer+1] x (the
 * split chosen for n_rows) x 4 bytes exceeds the array: fp32 storage always fits (256 x 256 weights over 32,768
 * or more rows use all of it); bf16 storage, whose tiles are twice as tall, fits up to half its full split
 * (512 x 512 weights: up to 8,447 rows). All calls on one GPU share
 * the array: calls that may overlap on the device (different streams, different contexts, different host threads)
 * race and must be ordered by the caller. Nothing in the array has to start at zero. The first call on a device
 * (or varco_prepare) looks the array's address up once; that first call is not capturable. Not bracketed by the
 * per-kernel profiler. */
int32_t varco_transform_bwd_weight_static(varco_ctx* ctx, int32_t layer, int64_t n_rows, const void* y, const void* dx_out,
                                          const void* x_out, void* dh, varco_stream stream);

/* Owner side of the backward exchange for partition p, all consumers at once (Section III: in the backward
 * pass the exchange runs from consumers to owners; Algorithm 1: errors cross machines): for every
 * boundary row b of p, v = its node id,
 *   dx_local[boundary_rows[b], pi_v(j)] += sum_{e in [ret_ptr[b], ret_ptr[b+1])} returned[ret_src[e], j],  j < k_layer
 * where `returned` holds rows of k_layer values (the consumers' dz_halo buffers, addressed as one array)
 * and ret_src lists, consumer partitions in ascending order, the rows that belong to b. The sum over
 * consumers is formed first, in that fixed order, then added to dx_local once. Equivalent to one
 * varco_decompress(accumulate = 1) per consumer, with a fraction of the memory traffic.
 * ret_ptr[n_boundary + 1], ret_src[ret_ptr[n_boundary]] device int32; dx_local n_local x width[layer].
 * ret_ptr = ret_src = NULL selects the map given at registration (STATE error when none was given). */
int32_t varco_accumulate_returned(varco_ctx* ctx, int32_t layer, int32_t p, const int32_t* ret_ptr,
                                  const int32_t* ret_src, const void* returned, void* dx_local,
                                  varco_stream stream);

int32_t varco_get_stats(const varco_ctx* ctx, varco_stats* out);
int32_t varco_reset_stats(varco_ctx* ctx);

/* ------------------------------------------------------------------------------------------------
 * Per-kernel timing for roofline reports (not part of the method). While enabled, every kernel launch of
 * the library is bracketed by a pair of HIP events on the launch stream. varco_profile_read synchronises
 * those events and returns, per kernel class, the number of launches, the summed duration in ms and the
 * summed algorithmic work of those launches: bytes the method itself must move (CSR entries and row
 * pointers, each local row once, each halo row once in compressed form, each output row once) for the
 * memory-bound classes, floating-point operations (2 m n k) for the matrix-core classes.
 */
enum {
    VARCO_K_COMPRESS = 0,       /* encoder: boundary rows -> k kept elements */
    VARCO_K_DECOMPRESS = 1,     /* decoder / owner-side accumulation of returned errors */
    VARCO_K_AGG_FWD = 2,        /* M = S_q [X_loc ; compressed halo] */
    VARCO_K_GEMM_FWD = 3,       /* act(M H1 + X H0) */
    VARCO_K_GEMM_WGRAD = 4,     /* dH += M^T dZ, X^T dZ (split reduction, partial products) */
    VARCO_K_GEMM_DGRAD = 5,     /* dM = dZ H1^T, dX += dZ H0^T */
    VARCO_K_AGG_BWD_LOCAL = 6,  /* dX_loc = S_loc^T dM */
    VARCO_K_AGG_BWD_HALO = 7,   /* dZ_halo = kept positions of S_halo^T dM (first pass: products in row order) */
    VARCO_K_REDUCE = 8,         /* fixed-order sums of split rows / split reductions */
    VARCO_K_AGG_BWD_HALO_SUM = 9, /* second pass of dZ_halo: sums of each halo row's products */
    VARCO_K_COUNT = 10
};
typedef struct {
    int64_t launches[VARCO_K_COUNT];
    double ms[VARCO_K_COUNT];
    double bytes[VARCO_K_COUNT];
    double flops[VARCO_K_COUNT];
    double stream_bytes[VARCO_K_COUNT];   /* the same launches' bytes when no cache serves a re-read: the gather kernels
                                           * (aggregation forward, transposed local block) fetch one source row per entry
                                           * instead of each row once; equal to bytes for the streaming kernels */
} varco_profile;
/* dst[i] += src[i] for n fp32 values (device pointers). Algorithm 1: the weight gradients computed on the
 * partitions are summed before the update; a caller that lets overlapping layer calls accumulate into one
 * gradient buffer per stream folds those buffers with this call. */
int32_t varco_sum_gradients(void* dst, const void* src, int64_t n, varco_stream stream);

/* ------------------------------------------------------------------------------------------------
 * The rest of Algorithm 1's iteration around the layer calls: loss, gradient step, rate schedule.
 */

/* Section II, the empirical risk with the cross-entropy as the loss, on the rows of one partition:
 *   loss_i = logsumexp(logits[i, :]) - logits[i, labels[i]]
 *   dlogits[i, :] = scale * (softmax(logits[i, :]) - onehot(labels[i]))
 * for rows with labels[i] in [0, n_classes); a row with labels[i] < 0 is not a training node: loss 0,
 * gradient 0 (a label >= n_classes is treated the same way and never used as an index). scale is 1 / (number of training nodes of the whole graph), so that the weight gradients
 * summed over partitions are those of the risk. Written: row_loss[n_rows] (fp32, unscaled), row_correct[n_rows]
 * (int32, 1 when the largest logit, lowest index on ties, is the label); when totals != NULL also
 * totals[0] += scale * sum(row_loss), totals[1] += sum(row_correct), summed in a fixed order (fp32[2]).
 * logits (leading dimension ld) and dlogits (ldd) have the context's storage type; dlogits may be NULL
 * (evaluation only). All pointers device. */
int32_t varco_softmax_xent(varco_ctx* ctx, const void* logits, int64_t ld, const int32_t* labels, int64_t n_rows,
                           int32_t n_classes, float scale, void* dlogits, int64_t ldd, float* row_loss,
                           int32_t* row_correct, float* totals, varco_stream stream);

/* The gradient step (SGD) of Section II: w[i] -= lr * dw[i] for n fp32 values (device pointers). Replicas
 * that start equal and take this step with the summed gradient stay equal, which is what Algorithm 1's
 * averaging of the workers' parameters amounts to. */
int32_t varco_sgd_step(void* w, const void* dw, int64_t n, float lr, varco_stream stream);

/* Section IV / Appendix "Scheduler": the compression ratio of iteration `step` of `n_steps`, as an exact
 * rational num/den >= 1 for varco_set_ratio (host only, no device work). The ratio starts at c_max and never
 * increases; it is clamped at c_min >= 1.
 *   VARCO_SCHED_LINEAR           max(c_max - param * (c_max - c_min) * step / n_steps, c_min), param = slope
 *   VARCO_SCHED_FIXED_INCREMENT  max(c_max - param * step, c_min), param = decrement per iteration
 *   VARCO_SCHED_EXPONENTIAL      clamp(param ^ (n_steps - step + 1), c_min, c_max), param = integer base >= 2
 * INVALID_ARG for c_min < 1, c_max < c_min, n_steps < 1, step < 0, a base < 2 or an unknown kind; SHAPE when
 * the rational does not fit 32 bits. */
enum { VARCO_SCHED_LINEAR = 0, VARCO_SCHED_FIXED_INCREMENT = 1, VARCO_SCHED_EXPONENTIAL = 2 };
int32_t varco_schedule_ratio(int32_t kind, int64_t step, int64_t n_steps, uint32_t c_max, uint32_t c_min,
                             uint32_t param, uint32_t* num, uint32_t* den);

/* A plain device-to-device copy of `bytes` bytes (multiple of 16, 16-byte aligned pointers) by a kernel
 * of this library: the known-size reference against which hardware byte counters are scaled. */
int32_t varco_calibration_copy(void* dst, const void* src, int64_t bytes, varco_stream stream);
int32_t varco_profile_enable(varco_ctx* ctx, int32_t on);
/* Synchronises the recorded events (blocks until the bracketed work has finished); reset != 0 clears the
 * totals afterwards. */
int32_t varco_profile_read(varco_ctx* ctx, varco_profile* out, int32_t reset);

#ifdef __cplusplus
}
#endif
#endif /* VARCO_H */
