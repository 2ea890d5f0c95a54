// Internal declarations shared by the translation units of libvarco (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <vector>

#include "varco.h"

// Brackets kernel launches with HIP events on the launch stream (see varco_profile_enable). When a launch
// follows the previous bracketed launch on the same stream, the previous stop event doubles as its start
// event: an event record is a marker in the queue that keeps the next kernel from starting early, so half as
// many markers disturb the run half as much.
struct VarcoProfiler {
    struct Rec {
        int cls;
        int start, stop;     // indices into `events`
        double bytes, flops;
        double stream_bytes;   // bytes when no cache serves a re-read (one source row per entry); = bytes for streaming kernels
    };
    bool on = false;
    std::vector<Rec> recs;
    std::vector<hipEvent_t> events;   // recorded since the last read
    std::vector<hipEvent_t> pool;     // free
    hipStream_t last_stream = nullptr;
    int last_stop = -1;               // event index of the last stop record, still the tail of last_stream's queue
    int record(hipStream_t st) {
        hipEvent_t e = nullptr;
        if (!pool.empty()) {
            e = pool.back();
            pool.pop_back();
        } else {
            (void)hipEventCreate(&e);
        }
        (void)hipEventRecord(e, st);
        events.push_back(e);
        return int(events.size()) - 1;
    }
    void begin(int cls, hipStream_t st, double bytes, double flops, double stream_bytes = -1.0) {
        if (!on) return;
        const int start = (last_stop >= 0 && last_stream == st) ? last_stop : record(st);
        recs.push_back(Rec{cls, start, -1, bytes, flops, stream_bytes < 0 ? bytes : stream_bytes});
        last_stop = -1;
    }
    void end(hipStream_t st) {
        if (!on) return;
        recs.back().stop = record(st);
        last_stream = st;
        last_stop = recs.back().stop;
    }
    // An untimed launch went to `st`: the next bracket on it needs a start event of its own.
    void interrupt() { last_stop = -1; }
};
// Work attributed to one launch, handed from the API layer to the launchers.
struct LaunchTag {
    VarcoProfiler* prof = nullptr;
    int cls = 0;
    double bytes = 0, flops = 0;
    double stream_bytes = -1;   // < 0: same as bytes
    void begin(hipStream_t st) const { if (prof) prof->begin(cls, st, bytes, flops, stream_bytes); }
    void begin_as(int other, hipStream_t st, double other_bytes) const { if (prof) prof->begin(other, st, other_bytes, 0); }
    void end(hipStream_t st) const { if (prof) prof->end(st); }
};

// Records `msg` as the last error of ctx (or of the process when ctx is null) and returns `code`.
int32_t varco_fail(const varco_ctx* ctx, int32_t code, const char* msg);

// The kept positions of a node vector (Definition 1 / Appendix A of the paper, with this library's keyed
// rule): pi_v(j) = (a_v * j + b_v) mod width, j < k, where b_v = floor(h1 * width / 2^32), a_v =
// units[floor(h2 * n_units / 2^32)], h1 = mix(v ^ s0), h2 = mix(h1 ^ s1), and (s0, s1) are derived on the
// host from (key, step, layer). k == width means the identity. Passed by value to kernels.
struct MaskRule {
    uint32_t s0, s1;
    uint32_t width, k;
    uint32_t n_units;
    uint32_t width_magic;       // floor(2^32 / width), 0xFFFFFFFF for width 1
    const uint16_t* units;      // device: ascending multipliers coprime with width
    const uint16_t* units_inv;  // device: their inverses modulo width
    const uint32_t* words;      // device, or null: when set, (s0, s1) are read from here instead (step table)
};

// One unit of SpMM work: entries [e0, e1) of CSR row `row`; dst < 0 writes the output row directly, else
// the partial sum goes to slot dst of the partial buffer (rows longer than the chunk length are split).
struct SpmmItem {
    int32_t row, e0, e1, dst;
};
// A split row and the contiguous range of partial slots that add up to it.
struct SpmmSplit {
    int32_t row, first, count, pad;
};
struct SpmmPlan {
    int32_t n_items = 0, n_splits = 0, n_partials = 0;
    // dense-only blocks with very short rows: rows short_r0 .. short_r0 + short_rows - 1 with at most short_max_len
    // entries are not on `items` but taken four to a wavefront, straight from the row pointer (device, borrowed)
    int32_t short_r0 = 0, short_rows = 0, short_max_len = 0;
    const int32_t* short_rowptr = nullptr;
    SpmmItem* items = nullptr;    // device
    SpmmSplit* splits = nullptr;  // device
};

// Per-entry record of a partition's row block, derived by the library at registration: a local column
// becomes {local row, -1}; a halo column becomes {row of that node in the concatenated compressed buffer,
// node id} (the id keys the node's kept positions).
struct VarcoEdge {
    int32_t src, gid;
};

// `dtype` (VARCO_F32 / VARCO_BF16) is the storage type of every activation, message and gradient buffer
// passed as void*; sums are formed in fp32 and rounded to nearest even on store.
hipError_t varco_launch_compress(int dtype, const MaskRule& rule, const int32_t* gids, const int32_t* rows, int64_t n_rows,
                                 const void* x, int64_t ldx, void* z, hipStream_t stream, const LaunchTag& tag);
hipError_t varco_launch_decompress(int dtype, const MaskRule& rule, const int32_t* gids, const int32_t* rows,
                                   int64_t n_rows, const void* z, void* x, int64_t ldx, int accumulate,
                                   hipStream_t stream, const LaunchTag& tag);

// x[rows[b], pi_v(j)] += sum_{e in [ptr[b], ptr[b+1])} returned[src[e] * k + j], v = gids[b].
hipError_t varco_launch_accumulate_returned(int dtype, const MaskRule& rule, const int32_t* gids, const int32_t* rows,
                                            int64_t n_rows, const int32_t* ptr, const int32_t* src, const void* returned,
                                            void* x, int64_t ldx, hipStream_t stream, const LaunchTag& tag);

hipError_t varco_launch_calibration_copy(void* dst, const void* src, int64_t bytes, hipStream_t stream);
hipError_t varco_launch_sum_gradients(float* dst, const float* src, int64_t n, hipStream_t stream);

// out[s] = {(a << 16) | b of node gids[s] under `rule` (1 << 16, the identity, when every element is kept), zrow[s]}:
// element j of halo row s sits at position (a j + b) mod width; the per-row records of HaloTransform.
hipError_t varco_launch_halo_rows(const MaskRule& rule, const int32_t* gids, const int32_t* zrow, int32_t n, uint2* out,
                                  hipStream_t stream);

// Device-resident step state: *d_step = the step (set to `value` when set != 0, else incremented), and
// table[2 t], table[2 t + 1] = the two key words of tap address t (0 .. 255) for that step and `key`.
hipError_t varco_launch_step_table(uint64_t* d_step, uint32_t* table, uint64_t key, int set, uint64_t value,
                                   hipStream_t stream);

// Index checks at registration: bits set in *flags (device int32, zeroed by the caller) by the first failed check
// of each kind.
enum {
    VARCO_BAD_COLUMN_RANGE = 1, VARCO_BAD_COLUMN_ORDER = 2, VARCO_BAD_TROW_RANGE = 4, VARCO_BAD_TROW_ORDER = 8,
    VARCO_BAD_TRANSPOSE = 16, VARCO_BAD_ID = 32, VARCO_BAD_BOUNDARY = 64, VARCO_BAD_RETURN_MAP = 128
};
hipError_t varco_launch_validate_partition(const varco_partition_desc& d, int32_t* flags, hipStream_t stream);

hipError_t varco_launch_build_edges(const int32_t* colidx, int64_t nnz, int32_t n_local, const int32_t* halo_zrow,
                                    const int32_t* halo_gid, VarcoEdge* edge, hipStream_t stream);

// out[row - row_base, :] = sum_e vals[e] * source_row(e) for the rows of `plan`, width = rule.width.
//   edge != null (forward): entry e reads dense + edge[e].src * width when edge[e].gid < 0, else the k kept
//       elements z[edge[e].src * k + j], which land at pi_gid(j) (a full row of z when k == width);
//   edge == null (transposed, all dense): entry e reads dense + colidx[e] * width.
// partial: workspace of plan.n_partials * width floats (fp32 for either storage type). z_rows: rows of z (0 when
// unknown); a compressed buffer below 4 GiB is addressed with 32-bit offsets.
hipError_t varco_launch_spmm(int dtype, const SpmmPlan& plan, const VarcoEdge* edge, const int32_t* colidx,
                             const float* vals, const void* dense, const void* z, int64_t z_rows, const MaskRule& rule,
                             void* out, int32_t row_base, float* partial, hipStream_t stream, const LaunchTag& tag);

// prow[e] = position of forward entry e among the halo entries of the transposed order (-1 for local entries).
hipError_t varco_launch_build_prow(const int32_t* rowptr, const int32_t* colidx, int32_t n_local,
                                   const int32_t* t_rowptr, const int32_t* t_colidx, int32_t* prow, hipStream_t stream);

// out[s, j] = sum over local rows i of S[i, halo s] * dm[i, pi_v(j)], j < k (the halo rows of the transposed
// aggregation, produced directly in compressed form) in two streaming passes through the product buffer
// `prod` ((halo entries) x k elements of the storage type). prod_base = transposed position of the first halo entry.
hipError_t varco_launch_halo_grad(int dtype, const SpmmPlan& fwd_plan, const SpmmPlan& t_halo_plan, const VarcoEdge* edge,
                                  const float* vals, const int32_t* prow, int32_t prod_base, const void* dm,
                                  const MaskRule& rule, void* prod, void* out, int32_t row_base, float* partial,
                                  hipStream_t stream, const LaunchTag& tag, const LaunchTag& sum_tag);

// C (+)= op(A) op(B) in fp32 on the matrix cores, row-major everywhere.
struct GemmOperand {
    const void* ptr = nullptr;    // matrix as stored
    const void* gate = nullptr;   // optional, same shape and type: elements are used only where gate > 0 (ReLU mask)
    int dtype = VARCO_F32;        // storage type of ptr and gate
    int64_t ld = 0;
    bool transposed = false;      // false: stored [rows=M or K][cols=K or N]; true: stored the other way round
};
struct GemmArgs {
    int32_t m = 0, n = 0, k = 0;
    GemmOperand a, b;             // first product
    GemmOperand a2, b2;           // optional second product summed into the same C (k2 reduction length)
    int32_t k2 = 0;
    // optional bf16 copies of B / B2 laid out [n][pitch] (reduction index contiguous, zero-padded to the pitch),
    // made by varco_launch_prep_weight: with them, bf16 activations go through the bf16 matrix-core kernel
    const void* b_prep = nullptr;
    const void* b2_prep = nullptr;
    int64_t b_prep_ld = 0, b2_prep_ld = 0;
    // fp32 operands on the bf16 matrix cores: 0 = no (fp32 matrix instructions); 2 or 3 = each operand is
    // expanded into that many bf16 terms, and b_prep / b2_prep are expanded copies made by
    // varco_launch_prep_weight_split, [term][n][pitch] with `plane` elements between terms
    int32_t f32_terms = 0;
    int64_t b_prep_plane = 0, b2_prep_plane = 0;
    void* c = nullptr;
    int c_dtype = VARCO_F32;
    int64_t ldc = 0;
    bool accumulate = false;      // C += instead of C =
    bool relu = false;            // C = max(., 0)
    int32_t split_k = 1;          // > 1: partial products into `partial` then reduced in a second kernel
    float* partial = nullptr;     // split_k * m * n floats
};
hipError_t varco_launch_gemm(const GemmArgs& g, hipStream_t stream, const LaunchTag& tag);
// c (+)= sum over s < slabs of partial[s][m x n], in a fixed order (the second pass of every split reduction).
hipError_t varco_launch_gemm_reduce(const float* partial, int32_t slabs, int32_t m, int32_t n, float* c, int64_t ldc,
                                    bool accumulate, hipStream_t stream, const LaunchTag& tag);

// The halo rows of a partition as an exchange delivered them (kernels_halo_transform.hip; bf16 storage): row s holds
// the k elements z[rec[s].y * k + j] at positions (a j + b) mod width, (a << 16) | b = rec[s].x, of a width-wide row
// that is zero elsewhere. width: a multiple of 16, at most 512; fo <= 64 columns on the other side of the weights.
struct HaloTransform {
    const void* z = nullptr;
    const uint2* rec = nullptr;
    int32_t n = 0;
    uint32_t width = 0, k = 0, width_magic = 0;
    int32_t fo = 0;
};
// y[s, :] = X~[s, :] H (n x fo, bf16), H as its bf16 copy wt[column][position] (pitch wpitch).
hipError_t varco_launch_halo_transform_fwd(const HaloTransform& h, const void* wt, int32_t wpitch, void* y, hipStream_t stream);
// dz[s, j] = (dy[s, :] H^T)[position of j] (n x k, bf16), H as its bf16 copy wr[position][column] (pitch cpitch).
hipError_t varco_launch_halo_transform_bwd(const HaloTransform& h, const void* dy, const void* wr, int32_t cpitch, void* dz,
                                           hipStream_t stream);
// partial[g][width x fo] = workgroup g's share of X~^T dy; *slabs = number of shares written (sum them with
// varco_launch_gemm_reduce). partial_elems: floats the buffer holds.
hipError_t varco_launch_halo_transform_wgrad(const HaloTransform& h, const void* dy, float* partial, int64_t partial_elems,
                                             int32_t* slabs, hipStream_t stream);

// bf16 matrix-core path (bf16 operands, fp32 accumulation). `usable` says whether the shapes, types and
// alignments of `g` fit it; the launcher runs the product kernel only and reports the number of reduction
// slabs it wrote to g.partial (1: the result is already in C).
bool varco_gemm_bf16_usable(const GemmArgs& g);
hipError_t varco_launch_gemm_bf16(const GemmArgs& g, hipStream_t stream, const LaunchTag& tag, int32_t* split_used);
// out[r][c] (bf16, row pitch `pitch` >= cols, zero beyond cols) = transpose ? h[c][r] : h[r][c] for r < rows.
hipError_t varco_launch_prep_weight(const float* h, int64_t ld, int32_t rows, int32_t cols, int32_t pitch, bool transpose,
                                    void* out, hipStream_t stream);

// fp32 operands as sums of bf16 terms on the bf16 matrix cores (kernels_gemm_split.hip); same contract as
// the bf16 path above.
bool varco_gemm_split_usable(const GemmArgs& g);
hipError_t varco_launch_gemm_split(const GemmArgs& g, hipStream_t stream, const LaunchTag& tag, int32_t* split_used);
// Expanded copy of (transpose ? h[c][r] : h[r][c]) (bf16 terms; rows padded to rows_padded, a multiple of 128, columns
// to pitch, a multiple of 32; zero beyond rows x cols), stored by row tile and stage of 32 columns as the product
// kernel fetches it (layout: kernels_gemm_split.hip). Same size as a plain [term][row][pitch] copy.
hipError_t varco_launch_prep_weight_split(int terms, const float* h, int64_t ld, int32_t rows, int32_t cols,
                                          int32_t rows_padded, int32_t pitch, bool transpose, void* out, hipStream_t stream);

// C (+)= A B^T with at most 64 reduction steps on the bf16 matrix units (terms: 1 for bf16 storage, 2 or 3 bf16 terms
// per fp32 operand); same operand contract as the fp32-instruction kernel of kernels_gemm.hip that it replaces.
hipError_t varco_launch_gemm_short_k(const GemmArgs& g, int terms, hipStream_t stream);

// Loss and update of a training iteration (kernels_train.hip). row_loss / row_correct: n_rows each; totals
// (2 floats) may be null.
hipError_t varco_launch_softmax_xent(int dtype, const void* logits, int64_t ld, const int32_t* labels, int64_t n_rows,
                                     int32_t n_classes, float scale, void* dlogits, int64_t ldd, float* row_loss,
                                     int32_t* row_correct, float* totals, hipStream_t stream);
hipError_t varco_launch_sgd(float* w, const float* dw, int64_t n, float lr, hipStream_t stream);
