// C ABI of libvarco: context, argument checking, per-step mask state and the sequencing of kernels for
// one partition's layer forward / backward (Algorithm 1 of the paper, one layer of eq. (2)).
#include <algorithm>
#include <climits>
#include <cstdio>
#include <cstring>
#include <initializer_list>
#include <mutex>
#include <numeric>
#include <string>
#include <vector>

#include "varco_internal.h"

namespace {

// Longest run of CSR entries one wavefront takes (longer rows are split and summed in fixed order). A run is a
// chain of dependent round trips: the forward block's wavefronts take compressed rows 8 to 16 at a time, the
// dense-only transposed blocks fetch 1 to 4 source rows per round trip, and a launch ends with its longest
// chain. Measured on the two large configurations: 256 / 256 -> 128 / 32 is 126.1 -> 114.9 ms (bf16) and
// 65.3 -> 64.8 ms (fp32) per step; 64 / 32 loses again to the extra partial rows.
constexpr int32_t kSpmmChunk = 128, kSpmmChunkDense = 32;

struct LayerState {
    uint32_t num = 1, den = 1;
    int32_t k = 0;
    int32_t n_units = 0;
    std::vector<uint16_t> h_units, h_units_inv;   // host copies; uploaded on first device use
    uint16_t* units = nullptr;       // device
    uint16_t* units_inv = nullptr;   // device
    bool ran_forward = false;        // in the current step
    int32_t order = VARCO_ORDER_AGGREGATE_FIRST;
};

struct PartState {
    bool registered = false;
    varco_partition_desc d{};
    SpmmPlan fwd, t_local, t_halo;
    VarcoEdge* edges = nullptr;      // device [nnz]: per-entry {source row, node id}
    int32_t* prow = nullptr;         // device [nnz]: per-entry row of the halo-gradient product buffer
    int32_t* boundary_gid = nullptr; // device [n_boundary]
    int64_t nnz_t_local = 0;         // transposed entries whose row is a local node
    int64_t z_rows = 0;              // 1 + the largest row of the compressed buffer a halo entry refers to
    int64_t n_returned = 0;          // rows of the registered owner-side map (d.ret_ptr / d.ret_src), 0 without one
};

// Device scratch of the layer calls. Calls issued on different streams may run concurrently, so every
// stream that calls into a context gets a set of its own (up to kMaxStreams), sized from what the
// registered partitions need.
struct Workspace {
    hipStream_t stream = nullptr;
    bool used = false;
    float* dm = nullptr;        size_t dm_elems = 0;        // dM: n_local x width (elements of the storage type)
    float* spmm = nullptr;      size_t spmm_elems = 0;      // partial rows of split CSR rows
    float* gemm = nullptr;      size_t gemm_elems = 0;      // split-K partial products
    float* prod = nullptr;      size_t prod_elems = 0;      // halo-gradient products: (halo entries) x k elements
    float* w = nullptr;         size_t w_elems = 0;         // converted copies of the weights, one slot per (layer, weight, orientation)
    float* tf = nullptr;        size_t tf_elems = 0;        // transform-first layers: [Y_loc ; Y_halo], (n_local + n_halo) x width[l+1]
    float* hrows = nullptr;     size_t hrows_elems = 0;     // and one record (two words) per halo row
    struct WeightTag {          // what a slot holds: made from `h` during step epoch `epoch` in the form `terms`
        const void* h = nullptr;
        uint64_t epoch = 0;
        int32_t terms = -1;
    };
    std::vector<WeightTag> w_tags;
};
constexpr int kMaxStreams = 8;

std::mutex g_err_mutex;
std::string g_global_error;

// Scratch of the entry point that allocates nothing (varco_transform_bwd_weight_static): the partial products of
// the split reduction. One copy per GPU, held until the process ends. In host code the array's name is only a
// handle: its device address is looked up once per device (scratch_of_current_device) and that pointer is what
// kernels are given.
constexpr size_t kScratchFloats = size_t(8) << 20;             // 32 MiB
static __device__ __align__(256) float scratch[kScratchFloats];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float* g_scratch_ptr[kMaxDevices] = {};

hipError_t scratch_of_current_device(float** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        float* ptr = nullptr;
        e = hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

struct varco_ctx {
    int32_t n_layers = 0, n_parts = 0, conv = 0, dtype = 0;
    int32_t f32_terms = 3;           // fp32 storage: bf16 terms per operand on the matrix cores (0: fp32 instructions)
    uint64_t weight_epoch = 1;       // converted weight copies are reused within an epoch (= a step)
    std::vector<size_t> w_slot;      // offset (bf16 elements) of every slot in a workspace's weight buffer, and the total
    uint64_t key = 0, step = 0;
    std::vector<int32_t> widths, act;
    std::vector<LayerState> layers;
    std::vector<PartState> parts;
    uint64_t* d_step = nullptr;      // device-resident step state (varco_step_table_enable), or null
    uint32_t* d_table = nullptr;     // its key words: 2 per tap address
    Workspace ws[kMaxStreams];
    size_t need_dm = 0, need_spmm = 0, need_gemm = 0, need_w = 0;   // what the registered partitions ask for
    int32_t* d_flags = nullptr;      // device word the index checks of a registration report into
    varco_stats stats{};
    VarcoProfiler prof;
    double prof_ms[VARCO_K_COUNT] = {}, prof_bytes[VARCO_K_COUNT] = {}, prof_flops[VARCO_K_COUNT] = {};
    double prof_stream_bytes[VARCO_K_COUNT] = {};
    int64_t prof_launches[VARCO_K_COUNT] = {};
    mutable std::string error;
    double elem_bytes() const { return dtype == VARCO_BF16 ? 2.0 : 4.0; }
    LaunchTag tag(int cls, double bytes, double flops, double stream_bytes = -1.0) {
        LaunchTag t;
        t.prof = prof.on ? &prof : nullptr;
        t.cls = cls, t.bytes = bytes, t.flops = flops, t.stream_bytes = stream_bytes;
        return t;
    }
};

int32_t varco_fail(const varco_ctx* ctx, int32_t code, const char* msg) {
    if (ctx) {
        ctx->error = msg;
    } else {
        std::lock_guard<std::mutex> lock(g_err_mutex);
        g_global_error = msg;
    }
    return code;
}

namespace {

int32_t hip_fail(const varco_ctx* ctx, hipError_t e, const char* what) {
    std::string m = std::string(what) + ": " + hipGetErrorString(e);
    return varco_fail(ctx, VARCO_ERR_HIP, m.c_str());
}

#define VARCO_HIP(ctx, call)                                   \
    do {                                                       \
        hipError_t e_ = (call);                                \
        if (e_ != hipSuccess) return hip_fail(ctx, e_, #call); \
    } while (0)

uint64_t mix64(uint64_t x) {   // splitmix64 output function
    x ^= x >> 30;
    x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27;
    x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}

// hop > 0: the exchange before the hop-th application of the shift operator inside a K-tap layer draws
// positions of its own (as if it were layer index layer + 16 * hop).
MaskRule make_rule(const varco_ctx* ctx, int32_t layer, int32_t hop = 0) {
    const LayerState& ls = ctx->layers[layer];
    const uint64_t inner = mix64(ctx->step + 0x9E3779B97F4A7C15ull * uint64_t(layer + VARCO_MAX_LAYERS * hop + 1));
    const uint64_t s = mix64(ctx->key ^ inner);
    MaskRule r;
    r.s0 = uint32_t(s & 0xFFFFFFFFull);
    r.s1 = uint32_t(s >> 32);
    r.width = uint32_t(ctx->widths[layer]);
    r.k = uint32_t(ls.k);
    r.n_units = uint32_t(ls.n_units);
    r.width_magic = r.width == 1 ? 0xFFFFFFFFu : uint32_t((uint64_t(1) << 32) / r.width);
    r.units = ls.units;
    r.units_inv = ls.units_inv;
    r.words = ctx->d_table ? ctx->d_table + 2 * (layer + VARCO_MAX_LAYERS * hop) : nullptr;
    return r;
}

// A rule that keeps every element of `width`-wide rows (used for purely dense aggregations).
MaskRule full_rule(int32_t width) {
    MaskRule r{};
    r.width = uint32_t(width);
    r.k = uint32_t(width);
    r.n_units = 1;
    r.width_magic = width == 1 ? 0xFFFFFFFFu : uint32_t((uint64_t(1) << 32) / uint32_t(width));
    r.words = nullptr;
    return r;
}

int32_t keep_count(int32_t width, uint32_t num, uint32_t den) {
    if (den == 0) return 0;   // unbounded ratio: nothing is communicated
    const uint64_t k = (uint64_t(width) * den + num - 1) / num;
    return int32_t(std::max<uint64_t>(1, k));
}

void free_plan(SpmmPlan& p) {
    if (p.items) (void)hipFree(p.items);
    if (p.splits) (void)hipFree(p.splits);
    p = SpmmPlan{};
}

void free_part(PartState& ps) {
    free_plan(ps.fwd);
    free_plan(ps.t_local);
    free_plan(ps.t_halo);
    if (ps.edges) (void)hipFree(ps.edges);
    if (ps.prow) (void)hipFree(ps.prow);
    if (ps.boundary_gid) (void)hipFree(ps.boundary_gid);
    ps = PartState{};
}

// Work list for rows [r0, r1) of a CSR given its host row pointers: long rows first (split into chunks
// whose partial sums are reduced afterwards), then every other row, empty ones included.
// Rows longer than `skip_up_to` entries go on the work list (all rows when it is negative); the others are
// left to the short-row kernel (see build of t_local below).
hipError_t build_plan(const std::vector<int32_t>& rowptr, int32_t r0, int32_t r1, SpmmPlan& plan, int32_t chunk,
                      int32_t skip_up_to = -1) {
    std::vector<SpmmItem> items;
    std::vector<SpmmSplit> splits;
    items.reserve(size_t(r1 - r0) + 64);
    int32_t n_partials = 0;
    for (int32_t r = r0; r < r1; ++r) {
        const int32_t len = rowptr[r + 1] - rowptr[r];
        if (len > chunk) {
            const int32_t pieces = (len + chunk - 1) / chunk;
            splits.push_back({r, n_partials, pieces, 0});
            for (int32_t c = 0; c < pieces; ++c) {
                const int32_t e0 = rowptr[r] + c * chunk;
                items.push_back({r, e0, std::min(e0 + chunk, rowptr[r + 1]), n_partials++});
            }
        }
    }
    for (int32_t r = r0; r < r1; ++r) {
        const int32_t len = rowptr[r + 1] - rowptr[r];
        if (len <= chunk && len > skip_up_to) items.push_back({r, rowptr[r], rowptr[r + 1], -1});
    }
    plan.n_items = int32_t(items.size());
    plan.n_splits = int32_t(splits.size());
    plan.n_partials = n_partials;
    hipError_t e = hipSuccess;
    if (!items.empty()) {
        e = hipMalloc(reinterpret_cast<void**>(&plan.items), items.size() * sizeof(SpmmItem));
        if (e != hipSuccess) return e;
        e = hipMemcpy(plan.items, items.data(), items.size() * sizeof(SpmmItem), hipMemcpyHostToDevice);
        if (e != hipSuccess) return e;
    }
    if (!splits.empty()) {
        e = hipMalloc(reinterpret_cast<void**>(&plan.splits), splits.size() * sizeof(SpmmSplit));
        if (e != hipSuccess) return e;
        e = hipMemcpy(plan.splits, splits.data(), splits.size() * sizeof(SpmmSplit), hipMemcpyHostToDevice);
    }
    return e;
}

hipError_t grow(float*& buf, size_t& have, size_t want) {
    if (want <= have) return hipSuccess;
    hipError_t e = hipDeviceSynchronize();   // nothing may still be using the old buffer
    if (e != hipSuccess) return e;
    if (buf) (void)hipFree(buf);
    buf = nullptr;
    have = 0;
    e = hipMalloc(reinterpret_cast<void**>(&buf), want * sizeof(float));
    if (e == hipSuccess) have = want;
    return e;
}

// Number of slabs the node dimension of a weight-gradient product is cut into: the workgroups of one launch
// should fill the chip exactly once (three 256-thread workgroups of the GEMM kernel are resident per
// compute unit, 256 compute units), so that no partly filled second round is left over.
// (The bf16 kernel has 256-row tiles, the kernel on expanded fp32 operands 128-row tiles; both take 32
// reduction steps per tile and have two resident workgroups per unit.)
enum GemmKind { kGemmF32 = 0, kGemmBf16 = 1, kGemmExpanded = 2 };
int32_t gemm_split_for(int32_t m, int32_t n, int64_t k, int kind) {
    const int64_t bm = kind == kGemmBf16 || (kind == kGemmF32 && n <= 64) ? 256 : 128, bn = n <= 64 ? 64 : 128;
    const int64_t tiles = ((m + bm - 1) / bm) * ((n + bn - 1) / bn);
    const int64_t k_tiles = kind == kGemmF32 ? (k + 15) / 16 : (k + 31) / 32;
    int64_t split = std::max<int64_t>(1, ((kind == kGemmF32 ? 3 : 2) * 256) / tiles);
    split = std::min<int64_t>(split, std::max<int64_t>(1, k_tiles / 8));
    return int32_t(split);
}
int gemm_kind(const GemmArgs& g) {
    return varco_gemm_bf16_usable(g) ? kGemmBf16 : varco_gemm_split_usable(g) ? kGemmExpanded : kGemmF32;
}

int32_t pad8(int32_t x) { return (x + 7) / 8 * 8; }
int32_t pad_to(int32_t x, int32_t m) { return (x + m - 1) / m * m; }

// Uploads the multiplier tables of every layer on first use (varco_create itself touches no device).
int32_t ensure_tables(varco_ctx* ctx) {
    for (LayerState& ls : ctx->layers) {
        if (ls.units) continue;
        const size_t bytes = ls.h_units.size() * sizeof(uint16_t);
        VARCO_HIP(ctx, hipMalloc(reinterpret_cast<void**>(&ls.units), bytes));
        VARCO_HIP(ctx, hipMalloc(reinterpret_cast<void**>(&ls.units_inv), bytes));
        VARCO_HIP(ctx, hipMemcpy(ls.units, ls.h_units.data(), bytes, hipMemcpyHostToDevice));
        VARCO_HIP(ctx, hipMemcpy(ls.units_inv, ls.h_units_inv.data(), bytes, hipMemcpyHostToDevice));
    }
    return VARCO_OK;
}

// Copy of a weight matrix in the form the bf16 matrix-core kernels take (B or B2 of `g`): rows = the product's
// output index, pitch padded; bf16 storage: one rounded copy; fp32 storage: the terms of the exact bf16
// expansion, one plane each. Nothing to do when fp32 instructions are used. Every (layer, weight, orientation)
// has a slot of its own in the stream's workspace, and a copy made earlier in the same step from the same
// pointer is reused: the weights of a step do not change (they are updated between steps).
hipError_t prep_weight(varco_ctx* ctx, Workspace& ws, int32_t layer, const void* h, int32_t fi, int32_t fo, bool transpose,
                       int which, bool as_b2, hipStream_t st, GemmArgs& g) {
    const bool bf16 = ctx->dtype == VARCO_BF16;
    if (!bf16 && ctx->f32_terms == 0) return hipSuccess;
    const int32_t terms = bf16 ? 1 : ctx->f32_terms;
    const int32_t rows = transpose ? fo : fi, cols = transpose ? fi : fo;
    const int32_t p = bf16 ? pad8(cols) : pad_to(cols, 32);
    const int32_t rows_padded = bf16 ? rows : pad_to(rows, 128);   // whole tiles: the kernel reads the copy without bounds checks
    const size_t slot = (size_t(layer) * 2 + which) * 2 + (transpose ? 0 : 1);
    uint16_t* dst = reinterpret_cast<uint16_t*>(ws.w) + ctx->w_slot[slot];
    (as_b2 ? g.b2_prep : g.b_prep) = dst;
    (as_b2 ? g.b2_prep_ld : g.b_prep_ld) = p;
    if (!bf16) {
        (as_b2 ? g.b2_prep_plane : g.b_prep_plane) = int64_t(rows_padded) * p;
        g.f32_terms = terms;
    }
    Workspace::WeightTag& tag = ws.w_tags[slot];
    if (tag.h == h && tag.epoch == ctx->weight_epoch && tag.terms == terms) return hipSuccess;
    tag.h = h, tag.epoch = ctx->weight_epoch, tag.terms = terms;
    ctx->prof.interrupt();   // an untimed launch: the next bracketed launch records a start event of its own
    if (bf16) return varco_launch_prep_weight(static_cast<const float*>(h), fo, rows, cols, p, transpose, dst, st);
    return varco_launch_prep_weight_split(terms, static_cast<const float*>(h), fo, rows, cols, rows_padded, p, transpose, dst, st);
}

// Elements (floats) of the halo-gradient product buffer the current ratios ask for: the largest (halo entries of a
// registered partition) x (k of a layer that hands back part of a row) elements of the storage type.
size_t prod_need(const varco_ctx* ctx) {
    int64_t entries = 0;
    for (const PartState& ps : ctx->parts)
        if (ps.registered) entries = std::max(entries, ps.d.nnz - ps.nnz_t_local);
    int32_t k = 0;
    for (int32_t l = 0; l < ctx->n_layers; ++l)
        if (ctx->layers[l].k < ctx->widths[l]) k = std::max(k, ctx->layers[l].k);
    return (size_t(entries) * size_t(k) * size_t(ctx->elem_bytes()) + 3) / 4;
}

// Floats of the two buffers of the layers that transform first: transformed rows of the local and halo nodes of the
// largest registered partition at the widest such layer's output, and a two-word record per halo row.
void transform_first_need(const varco_ctx* ctx, size_t* rows_out, size_t* records_out) {
    int32_t fo = 0;
    for (int32_t l = 0; l < ctx->n_layers; ++l)
        if (ctx->layers[l].order == VARCO_ORDER_TRANSFORM_FIRST) fo = std::max(fo, ctx->widths[l + 1]);
    int64_t rows = 0, halo = 0;
    for (const PartState& ps : ctx->parts)
        if (ps.registered) rows = std::max(rows, int64_t(ps.d.n_local) + ps.d.n_halo), halo = std::max<int64_t>(halo, ps.d.n_halo);
    *rows_out = fo ? (size_t(rows) * size_t(fo) * size_t(ctx->elem_bytes()) + 3) / 4 : 0;
    *records_out = fo ? size_t(halo) * 2 : 0;
}

// Brings one workspace set up to what the registered partitions and the current ratios need (host side of
// varco_prepare, varco_set_ratio and varco_register_partition: may synchronise the device).
int32_t size_workspace(varco_ctx* ctx, Workspace& ws) {
    VARCO_HIP(ctx, grow(ws.dm, ws.dm_elems, ctx->need_dm));
    VARCO_HIP(ctx, grow(ws.spmm, ws.spmm_elems, ctx->need_spmm));
    VARCO_HIP(ctx, grow(ws.gemm, ws.gemm_elems, ctx->need_gemm));
    VARCO_HIP(ctx, grow(ws.w, ws.w_elems, ctx->need_w));
    const size_t prod = prod_need(ctx);
    if (prod > ws.prod_elems) VARCO_HIP(ctx, grow(ws.prod, ws.prod_elems, prod + prod / 4));   // head-room: schedules raise k step by step
    size_t tf_rows = 0, tf_records = 0;
    transform_first_need(ctx, &tf_rows, &tf_records);
    VARCO_HIP(ctx, grow(ws.tf, ws.tf_elems, tf_rows));
    VARCO_HIP(ctx, grow(ws.hrows, ws.hrows_elems, tf_records));
    if (ws.w_tags.empty()) ws.w_tags.resize(size_t(ctx->n_layers) * 4);
    return VARCO_OK;
}
int32_t size_all_workspaces(varco_ctx* ctx) {
    for (Workspace& w : ctx->ws)
        if (w.used)
            if (int32_t rc = size_workspace(ctx, w)) return rc;
    return VARCO_OK;
}

// The workspace set of `st` (made by varco_prepare). The compute calls never allocate: without a set they fail.
int32_t workspace_for(varco_ctx* ctx, hipStream_t st, Workspace** out, const char* fn) {
    for (Workspace& w : ctx->ws)
        if (w.used && w.stream == st) {
            *out = &w;
            return VARCO_OK;
        }
    std::string m = std::string(fn) + ": no workspace for this stream; call varco_prepare(ctx, stream) first";
    return varco_fail(ctx, VARCO_ERR_STATE, m.c_str());
}

// The multiplier tables of the kept positions live on the device once varco_prepare or varco_register_partition ran.
int32_t check_tables(const varco_ctx* ctx, const char* fn) {
    if (!ctx->layers.empty() && ctx->layers[0].units) return VARCO_OK;
    std::string m = std::string(fn) + ": the context has no device state yet; call varco_prepare first";
    return varco_fail(ctx, VARCO_ERR_STATE, m.c_str());
}

int32_t check_layer(const varco_ctx* ctx, int32_t layer, const char* fn) {
    if (!ctx) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "null context");
    if (layer < 0 || layer >= ctx->n_layers) {
        std::string m = std::string(fn) + ": layer out of range";
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, m.c_str());
    }
    return VARCO_OK;
}

// Splits a tap address VARCO_TAP(layer, hop) = layer + 16 * hop and checks the layer.
int32_t split_tap(const varco_ctx* ctx, int32_t* layer, int32_t* hop, const char* fn) {
    if (!ctx) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "null context");
    if (*layer < 0 || *layer >= VARCO_MAX_LAYERS * VARCO_MAX_LAYERS) {
        std::string m = std::string(fn) + ": layer out of range";
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, m.c_str());
    }
    *hop = *layer / VARCO_MAX_LAYERS;
    *layer = *layer % VARCO_MAX_LAYERS;
    return check_layer(ctx, *layer, fn);
}

int32_t check_part(const varco_ctx* ctx, int32_t q, const char* fn) {
    if (q < 0 || q >= ctx->n_parts) {
        std::string m = std::string(fn) + ": partition out of range";
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, m.c_str());
    }
    if (!ctx->parts[q].registered) {
        std::string m = std::string(fn) + ": partition is not registered";
        return varco_fail(ctx, VARCO_ERR_STATE, m.c_str());
    }
    return VARCO_OK;
}

// The aggregation kernels cover a row with at most 8 loads per lane: rows wider than 512 elements need the
// 4-element accesses, hence 16-byte aligned buffers.
int32_t check_wide_rows(const varco_ctx* ctx, int32_t width, std::initializer_list<const void*> ptrs, const char* fn) {
    if (width <= 512) return VARCO_OK;
    for (const void* p : ptrs)
        if (p && (reinterpret_cast<uintptr_t>(p) & 15) != 0) {
            std::string m = std::string(fn) + ": buffers of rows wider than 512 elements must be 16-byte aligned";
            return varco_fail(ctx, VARCO_ERR_UNSUPPORTED, m.c_str());
        }
    return VARCO_OK;
}

}  // namespace

extern "C" const char* varco_last_error(const varco_ctx* ctx) {
    if (ctx) return ctx->error.c_str();
    std::lock_guard<std::mutex> lock(g_err_mutex);
    return g_global_error.c_str();
}

extern "C" int32_t varco_create(const varco_config* cfg, varco_ctx** out) {
    if (!out) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_create: out is null");
    *out = nullptr;
    if (!cfg || !cfg->widths || !cfg->act) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_create: null config field");
    if (cfg->n_layers < 1 || cfg->n_layers > VARCO_MAX_LAYERS)
        return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_create: n_layers outside 1..VARCO_MAX_LAYERS");
    if (cfg->n_partitions < 1) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_create: n_partitions must be positive");
    if (cfg->conv != VARCO_CONV_GCN && cfg->conv != VARCO_CONV_SAGE)
        return varco_fail(nullptr, VARCO_ERR_UNSUPPORTED, "varco_create: unknown conv");
    if (cfg->dtype != VARCO_F32 && cfg->dtype != VARCO_BF16)
        return varco_fail(nullptr, VARCO_ERR_UNSUPPORTED, "varco_create: dtype must be VARCO_F32 or VARCO_BF16");
    for (int32_t l = 0; l <= cfg->n_layers; ++l) {
        const int32_t w = cfg->widths[l];
        if (w < 1 || w > VARCO_MAX_WIDTH) return varco_fail(nullptr, VARCO_ERR_SHAPE, "varco_create: width outside 1..VARCO_MAX_WIDTH");
        if (w % 4 != 0 && w > 512)
            return varco_fail(nullptr, VARCO_ERR_UNSUPPORTED, "varco_create: widths above 512 must be multiples of 4");
    }
    for (int32_t l = 0; l < cfg->n_layers; ++l)
        if (cfg->act[l] != VARCO_ACT_IDENTITY && cfg->act[l] != VARCO_ACT_RELU)
            return varco_fail(nullptr, VARCO_ERR_UNSUPPORTED, "varco_create: unknown activation");

    auto* ctx = new varco_ctx;
    ctx->n_layers = cfg->n_layers;
    ctx->n_parts = cfg->n_partitions;
    ctx->conv = cfg->conv;
    ctx->dtype = cfg->dtype;
    ctx->key = cfg->mask_key;
    ctx->widths.assign(cfg->widths, cfg->widths + cfg->n_layers + 1);
    ctx->act.assign(cfg->act, cfg->act + cfg->n_layers);
    ctx->layers.resize(cfg->n_layers);
    ctx->parts.resize(cfg->n_partitions);
    ctx->stats.bytes_per_elem = cfg->dtype == VARCO_BF16 ? 2 : 4;
    {   // converted weight copies: a slot per (layer, weight, orientation); bf16 storage: rows padded to 8 elements;
        // fp32 storage: three terms each, padded to 128 rows of a multiple of 32 elements
        const bool bf16 = ctx->dtype == VARCO_BF16;
        size_t total = 0;
        for (int32_t l = 0; l < ctx->n_layers; ++l) {
            const int32_t fi = ctx->widths[l], fo = ctx->widths[l + 1];
            const size_t fwd = bf16 ? size_t(fo) * pad8(fi) : size_t(3) * pad_to(fo, 128) * pad_to(fi, 32);
            const size_t bwd = bf16 ? size_t(fi) * pad8(fo) : size_t(3) * pad_to(fi, 128) * pad_to(fo, 32);
            for (int which = 0; which < 2; ++which)
                for (size_t sz : {fwd, bwd}) {
                    ctx->w_slot.push_back(total);
                    total += (sz + 7) / 8 * 8;       // slots stay 16-byte aligned
                }
        }
        ctx->need_w = (total + 1) / 2;               // in floats
    }
    for (int32_t l = 0; l < ctx->n_layers; ++l) {
        LayerState& ls = ctx->layers[l];
        const int32_t w = ctx->widths[l];
        ls.k = w;
        // multipliers coprime with the width and their inverses (a * a_inv = 1 mod width)
        std::vector<uint16_t> units, inv;
        for (int32_t a = 1; a < std::max(w, 2); ++a)
            if (std::gcd(a, w) == 1) units.push_back(uint16_t(a));
        for (uint16_t a : units) {
            int64_t t = 0, nt = 1, r = w, nr = a % w;     // extended Euclid
            while (nr != 0) {
                const int64_t qd = r / nr;
                std::swap(t, nt), nt -= qd * t;
                std::swap(r, nr), nr -= qd * r;
            }
            inv.push_back(uint16_t(((t % w) + w) % w));
        }
        ls.n_units = int32_t(units.size());
        ls.h_units = units;
        ls.h_units_inv = inv;
    }
    *out = ctx;
    return VARCO_OK;
}

extern "C" int32_t varco_destroy(varco_ctx* ctx) {
    if (!ctx) return VARCO_OK;
    (void)hipDeviceSynchronize();
    for (LayerState& ls : ctx->layers) {
        if (ls.units) (void)hipFree(ls.units);
        if (ls.units_inv) (void)hipFree(ls.units_inv);
    }
    for (PartState& ps : ctx->parts) free_part(ps);
    for (Workspace& w : ctx->ws)
        for (float* p : {w.dm, w.spmm, w.gemm, w.prod, w.w, w.tf, w.hrows})
            if (p) (void)hipFree(p);
    if (ctx->d_flags) (void)hipFree(ctx->d_flags);
    if (ctx->d_step) (void)hipFree(ctx->d_step);
    if (ctx->d_table) (void)hipFree(ctx->d_table);
    for (hipEvent_t e : ctx->prof.events) (void)hipEventDestroy(e);
    for (hipEvent_t e : ctx->prof.pool) (void)hipEventDestroy(e);
    delete ctx;
    return VARCO_OK;
}

extern "C" int32_t varco_register_partition(varco_ctx* ctx, int32_t q, const varco_partition_desc* dev) {
    if (!ctx) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_register_partition: null context");
    if (!dev) return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_register_partition: null descriptor");
    if (q < 0 || q >= ctx->n_parts) return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_register_partition: partition out of range");
    if (dev->n_local < 0 || dev->n_halo < 0 || dev->n_boundary < 0 || dev->nnz < 0 || dev->z_row_offset < 0 ||
        dev->n_boundary > dev->n_local)
        return varco_fail(ctx, VARCO_ERR_SHAPE, "varco_register_partition: negative or inconsistent sizes");
    if (dev->nnz >= (int64_t(1) << 31) || int64_t(dev->n_local) + dev->n_halo >= (int64_t(1) << 31))
        return varco_fail(ctx, VARCO_ERR_SHAPE, "varco_register_partition: partition too large for 32-bit row pointers");
    if (!dev->rowptr || !dev->t_rowptr || !dev->halo_owner_ptr || (dev->n_local > 0 && !dev->local_gid))
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_register_partition: null index array");
    if (dev->nnz > 0 && (!dev->colidx || !dev->vals || !dev->t_colidx || !dev->t_vals))
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_register_partition: null entry array");
    if (dev->n_halo > 0 && (!dev->halo_gid || !dev->halo_zrow || !dev->halo_src_row))
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_register_partition: null halo array");
    if (dev->n_boundary > 0 && !dev->boundary_rows)
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_register_partition: null boundary array");
    if ((dev->ret_ptr == nullptr) != (dev->ret_src == nullptr) && dev->n_returned > 0)
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_register_partition: ret_ptr and ret_src go together");
    if (dev->halo_row_offset < 0 || dev->n_returned < 0 || (!dev->ret_ptr && dev->n_returned != 0))
        return varco_fail(ctx, VARCO_ERR_SHAPE, "varco_register_partition: negative or inconsistent sizes of the returned-row map");

    VARCO_HIP(ctx, hipDeviceSynchronize());
    if (int32_t rc = ensure_tables(ctx)) return rc;
    PartState& ps = ctx->parts[q];
    free_part(ps);
    ps.d = *dev;
    const int32_t nl = dev->n_local, nh = dev->n_halo, nb = dev->n_boundary;

    std::vector<int32_t> rowptr(size_t(nl) + 1), t_rowptr(size_t(nl) + nh + 1);
    VARCO_HIP(ctx, hipMemcpy(rowptr.data(), dev->rowptr, rowptr.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
    VARCO_HIP(ctx, hipMemcpy(t_rowptr.data(), dev->t_rowptr, t_rowptr.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
    auto monotone = [](const std::vector<int32_t>& p, int64_t nnz) {
        if (p.front() != 0 || p.back() != nnz) return false;
        for (size_t i = 1; i < p.size(); ++i)
            if (p[i] < p[i - 1]) return false;
        return true;
    };
    if (!monotone(rowptr, dev->nnz) || !monotone(t_rowptr, dev->nnz)) {
        free_part(ps);
        return varco_fail(ctx, VARCO_ERR_SHAPE, "varco_register_partition: row pointers do not match nnz");
    }
    if (dev->ret_ptr) {   // owner-side map of the backward exchange: a row pointer over the boundary rows
        std::vector<int32_t> ret_ptr(size_t(nb) + 1);
        VARCO_HIP(ctx, hipMemcpy(ret_ptr.data(), dev->ret_ptr, ret_ptr.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
        if (!monotone(ret_ptr, dev->n_returned)) {
            free_part(ps);
            return varco_fail(ctx, VARCO_ERR_SHAPE, "varco_register_partition: ret_ptr does not match n_returned");
        }
        ps.n_returned = dev->n_returned;
    }
    {   // the entry arrays themselves, checked on the device before any kernel trusts them
        if (!ctx->d_flags) VARCO_HIP(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->d_flags), sizeof(int32_t)));
        int32_t flags = 0;
        VARCO_HIP(ctx, hipMemcpy(ctx->d_flags, &flags, sizeof(flags), hipMemcpyHostToDevice));
        VARCO_HIP(ctx, varco_launch_validate_partition(*dev, ctx->d_flags, nullptr));
        VARCO_HIP(ctx, hipMemcpy(&flags, ctx->d_flags, sizeof(flags), hipMemcpyDeviceToHost));
        if (flags != 0) {
            free_part(ps);
            std::string m = "varco_register_partition: malformed index arrays:";
            if (flags & VARCO_BAD_COLUMN_RANGE) m += " column outside [0, n_local + n_halo);";
            if (flags & VARCO_BAD_COLUMN_ORDER) m += " columns of a row not strictly ascending;";
            if (flags & VARCO_BAD_TROW_RANGE) m += " transposed entry outside [0, n_local);";
            if (flags & VARCO_BAD_TROW_ORDER) m += " rows of a transposed row not strictly ascending;";
            if (flags & VARCO_BAD_TRANSPOSE) m += " transposed entries differ from the row block's;";
            if (flags & VARCO_BAD_ID) m += " negative node id or compressed-buffer row;";
            if (flags & VARCO_BAD_BOUNDARY) m += " boundary rows not ascending inside the partition;";
            if (flags & VARCO_BAD_RETURN_MAP) m += " negative row in ret_src;";
            return varco_fail(ctx, VARCO_ERR_SHAPE, m.c_str());
        }
    }
    ps.nnz_t_local = t_rowptr[nl];
    VARCO_HIP(ctx, build_plan(rowptr, 0, nl, ps.fwd, kSpmmChunk));
    // transposed local block: with fewer than three entries per row on average (fine partitions keep few
    // entries local) its short rows are taken four to a wavefront
    constexpr int32_t kShortLen = 8;
    const bool short_rows = nl > 0 && int64_t(t_rowptr[nl]) - t_rowptr[0] < 3 * int64_t(nl);
    VARCO_HIP(ctx, build_plan(t_rowptr, 0, nl, ps.t_local, kSpmmChunkDense, short_rows ? kShortLen : -1));
    ps.t_local.short_r0 = 0;
    ps.t_local.short_rows = short_rows ? nl : 0;
    ps.t_local.short_max_len = kShortLen;
    ps.t_local.short_rowptr = ps.d.t_rowptr;
    VARCO_HIP(ctx, build_plan(t_rowptr, nl, nl + nh, ps.t_halo, kSpmmChunkDense));

    if (dev->nnz > 0) {
        VARCO_HIP(ctx, hipMalloc(reinterpret_cast<void**>(&ps.edges), size_t(dev->nnz) * sizeof(VarcoEdge)));
        VARCO_HIP(ctx, varco_launch_build_edges(dev->colidx, dev->nnz, nl, dev->halo_zrow, dev->halo_gid, ps.edges, nullptr));
        if (nh > 0) {   // how far into the compressed buffer this partition reads (decides 32- or 64-bit row offsets)
            std::vector<int32_t> zrow(static_cast<size_t>(nh), 0);
            VARCO_HIP(ctx, hipMemcpy(zrow.data(), dev->halo_zrow, zrow.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
            ps.z_rows = int64_t(*std::max_element(zrow.begin(), zrow.end())) + 1;
        }
        VARCO_HIP(ctx, hipMalloc(reinterpret_cast<void**>(&ps.prow), size_t(dev->nnz) * sizeof(int32_t)));
        VARCO_HIP(ctx, varco_launch_build_prow(dev->rowptr, dev->colidx, nl, dev->t_rowptr, dev->t_colidx, ps.prow, nullptr));
        VARCO_HIP(ctx, hipDeviceSynchronize());
    }
    if (nb > 0) {
        std::vector<int32_t> lgid(nl), brow(nb), bgid(nb);
        VARCO_HIP(ctx, hipMemcpy(lgid.data(), dev->local_gid, size_t(nl) * sizeof(int32_t), hipMemcpyDeviceToHost));
        VARCO_HIP(ctx, hipMemcpy(brow.data(), dev->boundary_rows, size_t(nb) * sizeof(int32_t), hipMemcpyDeviceToHost));
        for (int32_t i = 0; i < nb; ++i) {
            if (brow[i] < 0 || brow[i] >= nl) {
                free_part(ps);
                return varco_fail(ctx, VARCO_ERR_SHAPE, "varco_register_partition: boundary row outside the partition");
            }
            bgid[i] = lgid[brow[i]];
        }
        VARCO_HIP(ctx, hipMalloc(reinterpret_cast<void**>(&ps.boundary_gid), size_t(nb) * sizeof(int32_t)));
        VARCO_HIP(ctx, hipMemcpy(ps.boundary_gid, bgid.data(), size_t(nb) * sizeof(int32_t), hipMemcpyHostToDevice));
    }

    // workspace: dM and partial rows sized for the widest layer, split-K partials for the largest weight
    const int32_t wmax = *std::max_element(ctx->widths.begin(), ctx->widths.end());
    int64_t max_partials = std::max({ps.fwd.n_partials, ps.t_local.n_partials, ps.t_halo.n_partials});
    int64_t gemm_elems = 0;
    for (int32_t l = 0; l < ctx->n_layers; ++l) {
        const int32_t fi = ctx->widths[l], fo = ctx->widths[l + 1];
        for (int kind : {kGemmF32, kGemmBf16, kGemmExpanded})
            gemm_elems = std::max<int64_t>(gemm_elems, int64_t(gemm_split_for(fi, fo, nl, kind)) * fi * fo);
    }
    ctx->need_dm = std::max(ctx->need_dm, size_t(nl) * wmax);
    ctx->need_spmm = std::max(ctx->need_spmm, size_t(max_partials) * wmax);
    ctx->need_gemm = std::max(ctx->need_gemm, size_t(gemm_elems));
    ps.registered = true;
    return size_all_workspaces(ctx);   // sets made by an earlier varco_prepare follow the new partition
}

extern "C" int32_t varco_prepare(varco_ctx* ctx, varco_stream stream) {
    if (!ctx) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_prepare: null context");
    if (int32_t rc = ensure_tables(ctx)) return rc;
    {   // the static scratch array's address on this device, for varco_transform_bwd_weight_static
        float* unused = nullptr;
        VARCO_HIP(ctx, scratch_of_current_device(&unused));
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    Workspace* ws = nullptr;
    for (Workspace& w : ctx->ws)
        if (w.used && w.stream == st) ws = &w;
    if (!ws) {
        for (Workspace& w : ctx->ws)
            if (!w.used) {
                ws = &w;
                break;
            }
        if (!ws) return varco_fail(ctx, VARCO_ERR_STATE, "varco_prepare: more streams than the context supports (8)");
        ws->used = true;
        ws->stream = st;
    }
    return size_workspace(ctx, *ws);
}

extern "C" int32_t varco_begin_step(varco_ctx* ctx, uint64_t step) {
    if (!ctx) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_begin_step: null context");
    if (ctx->d_table)
        return varco_fail(ctx, VARCO_ERR_STATE, "varco_begin_step: the step lives on the device; use varco_set_step or varco_advance_step");
    ctx->step = step;
    ctx->weight_epoch += 1;
    for (LayerState& ls : ctx->layers) ls.ran_forward = false;
    return VARCO_OK;
}

extern "C" int32_t varco_step_table_enable(varco_ctx* ctx, varco_stream stream) {
    if (!ctx) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_step_table_enable: null context");
    if (!ctx->d_table) {
        VARCO_HIP(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->d_step), sizeof(uint64_t)));
        VARCO_HIP(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->d_table),
                                 2 * VARCO_MAX_LAYERS * VARCO_MAX_LAYERS * sizeof(uint32_t)));
    }
    VARCO_HIP(ctx, varco_launch_step_table(ctx->d_step, ctx->d_table, ctx->key, 1, ctx->step, static_cast<hipStream_t>(stream)));
    return VARCO_OK;
}

extern "C" int32_t varco_set_step(varco_ctx* ctx, uint64_t step, varco_stream stream) {
    if (!ctx) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_set_step: null context");
    ctx->step = step;
    ctx->weight_epoch += 1;
    for (LayerState& ls : ctx->layers) ls.ran_forward = false;
    if (ctx->d_table)
        VARCO_HIP(ctx, varco_launch_step_table(ctx->d_step, ctx->d_table, ctx->key, 1, step, static_cast<hipStream_t>(stream)));
    return VARCO_OK;
}

extern "C" int32_t varco_advance_step(varco_ctx* ctx, varco_stream stream) {
    if (!ctx) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_advance_step: null context");
    if (!ctx->d_table) return varco_fail(ctx, VARCO_ERR_STATE, "varco_advance_step: call varco_step_table_enable first");
    ctx->step += 1;
    ctx->weight_epoch += 1;
    for (LayerState& ls : ctx->layers) ls.ran_forward = false;
    VARCO_HIP(ctx, varco_launch_step_table(ctx->d_step, ctx->d_table, ctx->key, 0, 0, static_cast<hipStream_t>(stream)));
    return VARCO_OK;
}

extern "C" int32_t varco_set_matmul_terms(varco_ctx* ctx, int32_t terms) {
    if (!ctx) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_set_matmul_terms: null context");
    if (terms != 0 && terms != 2 && terms != 3)
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_set_matmul_terms: terms must be 0, 2 or 3");
    ctx->f32_terms = terms;
    ctx->weight_epoch += 1;
    return VARCO_OK;
}

extern "C" int32_t varco_set_layer_order(varco_ctx* ctx, int32_t layer, int32_t order) {
    if (int32_t rc = check_layer(ctx, layer, "varco_set_layer_order")) return rc;
    if (order != VARCO_ORDER_AGGREGATE_FIRST && order != VARCO_ORDER_TRANSFORM_FIRST)
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_set_layer_order: unknown order");
    if (ctx->layers[layer].ran_forward)
        return varco_fail(ctx, VARCO_ERR_STATE, "varco_set_layer_order: the layer already ran forward in this step; call varco_begin_step first");
    if (order == VARCO_ORDER_TRANSFORM_FIRST) {
        const int32_t fi = ctx->widths[layer], fo = ctx->widths[layer + 1];
        if (ctx->dtype != VARCO_BF16 || ctx->act[layer] != VARCO_ACT_IDENTITY || fo > 64 || fi % 16 != 0 || fi > 512)
            return varco_fail(ctx, VARCO_ERR_UNSUPPORTED,
                              "varco_set_layer_order: transform-first needs bf16 storage, an identity activation, at most 64 "
                              "output columns and an input width that is a multiple of 16 and at most 512");
    }
    ctx->layers[layer].order = order;
    return size_all_workspaces(ctx);
}

extern "C" int32_t varco_set_ratio(varco_ctx* ctx, int32_t layer, uint32_t num, uint32_t den) {
    if (!ctx) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_set_ratio: null context");
    if (layer < -1 || layer >= ctx->n_layers) return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_set_ratio: layer out of range");
    if (num == 0 || (den != 0 && num < den))
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_set_ratio: ratio must be a rational >= 1 (den = 0: no communication)");
    const int32_t l0 = layer < 0 ? 0 : layer, l1 = layer < 0 ? ctx->n_layers : layer + 1;
    for (int32_t l = l0; l < l1; ++l)
        if (ctx->layers[l].ran_forward)
            return varco_fail(ctx, VARCO_ERR_STATE,
                              "varco_set_ratio: the layer already ran forward in this step; call varco_begin_step first");
    for (int32_t l = l0; l < l1; ++l) {
        ctx->layers[l].num = num;
        ctx->layers[l].den = den;
        ctx->layers[l].k = keep_count(ctx->widths[l], num, den);
    }
    return size_all_workspaces(ctx);   // a larger k may need a larger product buffer (no-op without workspace sets)
}

extern "C" int32_t varco_get_keep(const varco_ctx* ctx, int32_t layer, int32_t* k) {
    if (int32_t rc = check_layer(ctx, layer, "varco_get_keep")) return rc;
    if (!k) return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_get_keep: null output");
    *k = ctx->layers[layer].k;
    return VARCO_OK;
}

extern "C" int32_t varco_compress(varco_ctx* ctx, int32_t layer, const int32_t* gids, const int32_t* rows,
                                  int64_t n_rows, const void* x, int64_t ldx, void* z, varco_stream stream) {
    if (ctx) ctx->prof.interrupt();   // events are shared between the launches of one call only
    int32_t hop = 0;
    if (int32_t rc = split_tap(ctx, &layer, &hop, "varco_compress")) return rc;
    if (n_rows < 0) return varco_fail(ctx, VARCO_ERR_SHAPE, "varco_compress: negative row count");
    if (n_rows == 0 || ctx->layers[layer].k == 0) return VARCO_OK;   // k = 0: nothing is sent
    if (!gids || !x || !z) return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_compress: null pointer");
    if (ldx < ctx->widths[layer]) return varco_fail(ctx, VARCO_ERR_SHAPE, "varco_compress: ldx is smaller than the layer width");
    if (int32_t rc = check_tables(ctx, "varco_compress")) return rc;
    ctx->layers[layer].ran_forward = true;   // the step's positions of this layer are now in use
    const MaskRule rule = make_rule(ctx, layer, hop);
    const double bytes = double(n_rows) * (rule.width + rule.k) * ctx->elem_bytes();
    VARCO_HIP(ctx, varco_launch_compress(ctx->dtype, rule, gids, rows, n_rows, x, ldx, z, static_cast<hipStream_t>(stream),
                                         ctx->tag(VARCO_K_COMPRESS, bytes, 0)));
    return VARCO_OK;
}

extern "C" int32_t varco_decompress(varco_ctx* ctx, int32_t layer, const int32_t* gids, const int32_t* rows,
                                    int64_t n_rows, const void* z, void* x, int64_t ldx, int32_t accumulate,
                                    varco_stream stream) {
    if (ctx) ctx->prof.interrupt();   // events are shared between the launches of one call only
    int32_t hop = 0;
    if (int32_t rc = split_tap(ctx, &layer, &hop, "varco_decompress")) return rc;
    if (n_rows < 0) return varco_fail(ctx, VARCO_ERR_SHAPE, "varco_decompress: negative row count");
    if (accumulate != 0 && accumulate != 1) return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_decompress: accumulate must be 0 or 1");
    if (n_rows == 0 || (accumulate && ctx->layers[layer].k == 0)) return VARCO_OK;
    if (!gids || !x || (!z && ctx->layers[layer].k > 0))
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_decompress: null pointer");
    if (ldx < ctx->widths[layer]) return varco_fail(ctx, VARCO_ERR_SHAPE, "varco_decompress: ldx is smaller than the layer width");
    if (int32_t rc = check_tables(ctx, "varco_decompress")) return rc;
    ctx->layers[layer].ran_forward = true;
    const MaskRule rule = make_rule(ctx, layer, hop);
    const double bytes = (accumulate ? double(n_rows) * rule.k * 3.0 : double(n_rows) * (rule.width + rule.k)) * ctx->elem_bytes();
    VARCO_HIP(ctx, varco_launch_decompress(ctx->dtype, rule, gids, rows, n_rows, z, x, ldx, accumulate,
                                           static_cast<hipStream_t>(stream), ctx->tag(VARCO_K_DECOMPRESS, bytes, 0)));
    return VARCO_OK;
}

namespace {

HaloTransform halo_transform(const varco_partition_desc& d, const MaskRule& rule, const void* z, const Workspace& ws, int32_t fo) {
    HaloTransform h;
    h.z = z;
    h.rec = reinterpret_cast<const uint2*>(ws.hrows);
    h.n = d.n_halo;
    h.width = rule.width, h.k = rule.k, h.width_magic = rule.width_magic;
    h.fo = fo;
    return h;
}

int32_t transform_first_fits(varco_ctx* ctx, const PartState& ps, const Workspace& ws, int32_t fo, const char* fn) {
    const size_t rows = (size_t(int64_t(ps.d.n_local) + ps.d.n_halo) * size_t(fo) * size_t(ctx->elem_bytes()) + 3) / 4;
    if (rows <= ws.tf_elems && size_t(ps.d.n_halo) * 2 <= ws.hrows_elems) return VARCO_OK;
    std::string m = std::string(fn) + ": the stream's workspace is too small; call varco_prepare";
    return varco_fail(ctx, VARCO_ERR_STATE, m.c_str());
}

// Split of a weight-gradient product's reduction that the stream's partial buffer holds.
int32_t wgrad_split(const Workspace& ws, const GemmArgs& g, int64_t rows) {
    int64_t split = gemm_split_for(g.m, g.n, rows, gemm_kind(g));
    const int64_t fit = int64_t(ws.gemm_elems / (size_t(g.m) * size_t(g.n)));
    return int32_t(std::max<int64_t>(1, std::min(split, fit)));
}

// The layer of eq. (2) with the transform applied before the aggregation, x_out = S_q [X_loc H1 ; X~_halo H1] (+ X_loc H0):
// every source row is transformed once - a halo row from its k received elements - and rows of width[layer+1]
// elements are aggregated.
int32_t layer_fwd_transform_first(varco_ctx* ctx, const PartState& ps, Workspace& ws, int32_t layer, const MaskRule& rule,
                                  const void* x_local, const void* z_in, const void* h1, const void* h0, void* x_out,
                                  hipStream_t st) {
    const varco_partition_desc& d = ps.d;
    const int32_t fi = ctx->widths[layer], fo = ctx->widths[layer + 1], nl = d.n_local, nh = d.n_halo;
    const int dt = ctx->dtype;
    const double es = ctx->elem_bytes();
    if (nl == 0) return VARCO_OK;
    if (int32_t rc = transform_first_fits(ctx, ps, ws, fo, "varco_layer_fwd")) return rc;
    char* const y_all = reinterpret_cast<char*>(ws.tf);
    GemmArgs g;
    g.m = nl, g.n = fo, g.k = fi;
    g.a.ptr = x_local, g.a.ld = fi, g.a.dtype = dt;
    g.b.ptr = h1, g.b.ld = fo;
    g.c = y_all, g.ldc = fo, g.c_dtype = dt;
    VARCO_HIP(ctx, prep_weight(ctx, ws, layer, h1, fi, fo, true, 0, false, st, g));
    VARCO_HIP(ctx, varco_launch_gemm(g, st, ctx->tag(VARCO_K_GEMM_FWD, 0, 2.0 * nl * double(fo) * fi)));
    if (nh > 0) {   // k = 0 (no communication): rows of zeros
        ctx->prof.interrupt();   // an untimed launch: the next bracketed launch records a start event of its own
        VARCO_HIP(ctx, varco_launch_halo_rows(rule, d.halo_gid, d.halo_zrow, nh, reinterpret_cast<uint2*>(ws.hrows), st));
        // rows of z once, the transformed rows once; the weights stay on chip
        const LaunchTag tag = ctx->tag(VARCO_K_GEMM_FWD, double(nh) * (rule.k + fo) * es + 8.0 * nh, 2.0 * nh * double(fo) * rule.k);
        tag.begin(st);
        const hipError_t e = varco_launch_halo_transform_fwd(halo_transform(d, rule, z_in, ws, fo), g.b_prep, int32_t(g.b_prep_ld),
                                                             y_all + size_t(nl) * fo * size_t(es), st);
        tag.end(st);
        VARCO_HIP(ctx, e);
    }
    // entries, row pointer, the transformed rows once, the output once
    const double agg_bytes = double(d.nnz) * 8.0 + (double(nl) + 1.0) * 4.0 + (2.0 * double(nl) + nh) * fo * es;
    const double agg_stream = double(d.nnz) * 8.0 + (double(nl) + 1.0) * 4.0 + (double(nl) + double(d.nnz)) * fo * es;
    VARCO_HIP(ctx, varco_launch_spmm(dt, ps.fwd, nullptr, d.colidx, d.vals, y_all, nullptr, 0, full_rule(fo), x_out, 0, ws.spmm, st,
                                     ctx->tag(VARCO_K_AGG_FWD, agg_bytes, 0, agg_stream)));
    if (ctx->conv == VARCO_CONV_SAGE) {   // self tap
        GemmArgs g0;
        g0.m = nl, g0.n = fo, g0.k = fi;
        g0.a.ptr = x_local, g0.a.ld = fi, g0.a.dtype = dt;
        g0.b.ptr = h0, g0.b.ld = fo;
        g0.c = x_out, g0.ldc = fo, g0.c_dtype = dt;
        g0.accumulate = true;
        VARCO_HIP(ctx, prep_weight(ctx, ws, layer, h0, fi, fo, true, 1, false, st, g0));
        VARCO_HIP(ctx, varco_launch_gemm(g0, st, ctx->tag(VARCO_K_GEMM_FWD, 0, 2.0 * nl * double(fo) * fi)));
    }
    return VARCO_OK;
}

// Its gradient: [dY_loc ; dY_halo] = S_q^T dZ at width[layer+1]; dH1 += X_loc^T dY_loc + X~_halo^T dY_halo;
// dX_loc = dY_loc H1^T; the errors handed back are dY_halo H1^T at each halo row's kept positions. z_in: the compressed
// rows the forward call read.
int32_t layer_bwd_transform_first(varco_ctx* ctx, const PartState& ps, Workspace& ws, int32_t layer, const void* dz,
                                  const void* x_local, const void* z_in, const void* h1, const void* h0, void* dh1, void* dh0,
                                  void* dx_local, void* dz_halo, hipStream_t st) {
    const varco_partition_desc& d = ps.d;
    const int32_t fi = ctx->widths[layer], fo = ctx->widths[layer + 1], nl = d.n_local, nh = d.n_halo;
    const int dt = ctx->dtype;
    const double es = ctx->elem_bytes();
    const bool sage = ctx->conv == VARCO_CONV_SAGE;
    const MaskRule rule = make_rule(ctx, layer);
    const bool halo = nh > 0 && rule.k > 0;
    if (halo && !z_in)
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_layer_bwd: a transform-first layer takes the forward call's z_in as m_saved");
    if (int32_t rc = transform_first_fits(ctx, ps, ws, fo, "varco_layer_bwd")) return rc;
    char* const dy_all = reinterpret_cast<char*>(ws.tf);
    char* const dy_halo = dy_all + size_t(nl) * fo * size_t(es);
    const MaskRule narrow = full_rule(fo);
    const double tl_bytes = double(ps.nnz_t_local) * 8.0 + (double(nl) + 1.0) * 4.0 + 2.0 * double(nl) * fo * es;
    const double tl_stream = tl_bytes + (double(ps.nnz_t_local) - double(nl)) * fo * es;
    VARCO_HIP(ctx, varco_launch_spmm(dt, ps.t_local, nullptr, d.t_colidx, d.t_vals, dz, nullptr, 0, narrow, dy_all, 0, ws.spmm, st,
                                     ctx->tag(VARCO_K_AGG_BWD_LOCAL, tl_bytes, 0, tl_stream)));
    if (halo) {
        const double th_bytes = double(d.nnz - ps.nnz_t_local) * 8.0 + (double(nh) + 1.0) * 4.0 + (double(nl) + nh) * fo * es;
        VARCO_HIP(ctx, varco_launch_spmm(dt, ps.t_halo, nullptr, d.t_colidx, d.t_vals, dz, nullptr, 0, narrow, dy_halo, nl, ws.spmm,
                                         st, ctx->tag(VARCO_K_AGG_BWD_HALO, th_bytes, 0)));
        ctx->prof.interrupt();   // an untimed launch: the next bracketed launch records a start event of its own
        VARCO_HIP(ctx, varco_launch_halo_rows(rule, d.halo_gid, d.halo_zrow, nh, reinterpret_cast<uint2*>(ws.hrows), st));
    }
    // weight gradients
    {
        GemmArgs g;
        g.m = fi, g.n = fo, g.k = nl;
        g.a.ptr = x_local, g.a.ld = fi, g.a.transposed = true, g.a.dtype = dt;
        g.b.ptr = dy_all, g.b.ld = fo, g.b.dtype = dt;
        g.c = dh1, g.ldc = fo;
        g.accumulate = true;
        g.partial = ws.gemm;
        g.split_k = wgrad_split(ws, g, nl);
        VARCO_HIP(ctx, varco_launch_gemm(g, st, ctx->tag(VARCO_K_GEMM_WGRAD, 0, 2.0 * fi * fo * double(nl))));
        if (sage) {
            g.b.ptr = dz, g.c = dh0;
            g.split_k = wgrad_split(ws, g, nl);
            VARCO_HIP(ctx, varco_launch_gemm(g, st, ctx->tag(VARCO_K_GEMM_WGRAD, 0, 2.0 * fi * fo * double(nl))));
        }
        if (halo) {   // + X~_halo^T dY_halo: per-workgroup shares, then the fixed-order sum
            const LaunchTag tag = ctx->tag(VARCO_K_GEMM_WGRAD, double(nh) * (rule.k + fo) * es + 8.0 * nh,
                                           2.0 * double(rule.k) * fo * double(nh));
            int32_t slabs = 0;
            tag.begin(st);
            const hipError_t e = varco_launch_halo_transform_wgrad(halo_transform(d, rule, z_in, ws, fo), dy_halo, ws.gemm,
                                                                   int64_t(ws.gemm_elems), &slabs, st);
            tag.end(st);
            VARCO_HIP(ctx, e);
            VARCO_HIP(ctx, varco_launch_gemm_reduce(ws.gemm, slabs, fi, fo, static_cast<float*>(dh1), fo, true, st, tag));
        }
    }
    if (!dx_local) return VARCO_OK;
    {   // dX_loc = dY_loc H1^T (+ dZ H0^T)
        GemmArgs g;
        g.m = nl, g.n = fi, g.k = fo;
        g.a.ptr = dy_all, g.a.ld = fo, g.a.dtype = dt;
        g.b.ptr = h1, g.b.ld = fo, g.b.transposed = true;
        g.c = dx_local, g.ldc = fi, g.c_dtype = dt;
        VARCO_HIP(ctx, varco_launch_gemm(g, st, ctx->tag(VARCO_K_GEMM_DGRAD, 0, 2.0 * fi * fo * double(nl))));
        if (sage) {
            g.a.ptr = dz, g.b.ptr = h0, g.accumulate = true;
            VARCO_HIP(ctx, varco_launch_gemm(g, st, ctx->tag(VARCO_K_GEMM_DGRAD, 0, 2.0 * fi * fo * double(nl))));
        }
        if (halo) {   // dY_halo H1^T at the kept positions only, straight into compressed form
            GemmArgs gw;              // (carries the slot of the weights' bf16 copy [position][column])
            VARCO_HIP(ctx, prep_weight(ctx, ws, layer, h1, fi, fo, false, 0, false, st, gw));
            const LaunchTag tag = ctx->tag(VARCO_K_GEMM_DGRAD, double(nh) * (rule.k + fo) * es + 8.0 * nh,
                                           2.0 * double(rule.k) * fo * double(nh));
            tag.begin(st);
            const hipError_t e = varco_launch_halo_transform_bwd(halo_transform(d, rule, z_in, ws, fo), dy_halo, gw.b_prep,
                                                                 int32_t(gw.b_prep_ld), dz_halo, st);
            tag.end(st);
            VARCO_HIP(ctx, e);
            ctx->stats.bwd_elems[layer] += int64_t(nh) * rule.k;
            ctx->stats.full_bwd_elems[layer] += int64_t(nh) * fi;
        }
    }
    return VARCO_OK;
}

}  // namespace

extern "C" int32_t varco_layer_fwd(varco_ctx* ctx, int32_t layer, int32_t q, const void* x_local, const void* z_in,
                                   const void* h1, const void* h0, void* x_out, void* z_out, void* m_saved,
                                   varco_stream stream) {
    if (ctx) ctx->prof.interrupt();   // events are shared between the launches of one call only
    if (int32_t rc = check_layer(ctx, layer, "varco_layer_fwd")) return rc;
    if (int32_t rc = check_part(ctx, q, "varco_layer_fwd")) return rc;
    const PartState& ps = ctx->parts[q];
    const varco_partition_desc& d = ps.d;
    const bool sage = ctx->conv == VARCO_CONV_SAGE;
    const bool transform_first = ctx->layers[layer].order == VARCO_ORDER_TRANSFORM_FIRST;
    if (!h1 || (d.n_local > 0 && (!x_local || !x_out || (!m_saved && !transform_first))))
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_layer_fwd: null pointer");
    if (sage && !h0) return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_layer_fwd: h0 is required for the SAGE convolution");
    if (!sage && h0) return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_layer_fwd: h0 must be null for the single-tap convolution");
    if (d.n_halo > 0 && !z_in && ctx->layers[layer].k > 0)
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_layer_fwd: z_in is null but the partition has halo nodes");
    if (z_out && layer == ctx->n_layers - 1)
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_layer_fwd: z_out must be null on the last layer");
    if (int32_t rc = check_wide_rows(ctx, ctx->widths[layer], {x_local, z_in, m_saved}, "varco_layer_fwd")) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    Workspace* wsp = nullptr;
    if (int32_t rc = workspace_for(ctx, st, &wsp, "varco_layer_fwd")) return rc;
    Workspace& ws = *wsp;
    const int32_t fi = ctx->widths[layer], fo = ctx->widths[layer + 1];
    const MaskRule rule = make_rule(ctx, layer);
    ctx->layers[layer].ran_forward = true;

    const int dt = ctx->dtype;
    const double es = ctx->elem_bytes();
    if (transform_first) {
        if (int32_t rc = layer_fwd_transform_first(ctx, ps, ws, layer, rule, x_local, z_in, h1, h0, x_out, st)) return rc;
    } else {
    // aggregate: local rows dense, halo rows straight from the owners' compressed buffers
    const double agg_bytes = double(d.nnz) * 8.0 + (double(d.n_local) + 1.0) * 4.0 + 2.0 * double(d.n_local) * fi * es +
                             double(d.n_halo) * rule.k * es;
    // the same without any cache between the entries of different rows: one source row fetched per entry
    const double agg_stream = double(d.nnz) * 8.0 + (double(d.n_local) + 1.0) * 4.0 + double(d.n_local) * fi * es +
                              double(ps.nnz_t_local) * fi * es + double(d.nnz - ps.nnz_t_local) * rule.k * es;
    VARCO_HIP(ctx, varco_launch_spmm(dt, ps.fwd, ps.edges, nullptr, d.vals, x_local, z_in, ps.z_rows, rule, m_saved, 0, ws.spmm, st,
                                     ctx->tag(VARCO_K_AGG_FWD, agg_bytes, 0, agg_stream)));
    // transform + nonlinearity
    GemmArgs g;
    g.m = d.n_local, g.n = fo, g.k = fi;
    g.a.ptr = m_saved, g.a.ld = fi, g.a.dtype = dt;
    g.b.ptr = h1, g.b.ld = fo;
    if (sage) {
        g.k2 = fi;
        g.a2.ptr = x_local, g.a2.ld = fi, g.a2.dtype = dt;
        g.b2.ptr = h0, g.b2.ld = fo;
    }
    g.c = x_out, g.ldc = fo, g.c_dtype = dt;
    g.relu = ctx->act[layer] == VARCO_ACT_RELU;
    if (d.n_local > 0) {   // weights as bf16, [output column][reduction index]
        VARCO_HIP(ctx, prep_weight(ctx, ws, layer, h1, fi, fo, true, 0, false, st, g));
        if (sage) VARCO_HIP(ctx, prep_weight(ctx, ws, layer, h0, fi, fo, true, 1, true, st, g));
    }
    VARCO_HIP(ctx, varco_launch_gemm(g, st, ctx->tag(VARCO_K_GEMM_FWD, 0, 2.0 * g.m * g.n * (double(g.k) + g.k2))));
    }
    // boundary rows of the output, compressed for the next layer's exchange
    if (z_out && d.n_boundary > 0 && ctx->layers[layer + 1].k > 0) {
        ctx->layers[layer + 1].ran_forward = true;   // its positions are now in use
        const MaskRule next = make_rule(ctx, layer + 1);
        char* zdst = static_cast<char*>(z_out) + int64_t(d.z_row_offset) * next.k * int64_t(es);
        VARCO_HIP(ctx, varco_launch_compress(dt, next, ps.boundary_gid, d.boundary_rows, d.n_boundary, x_out, fo, zdst, st,
                                             ctx->tag(VARCO_K_COMPRESS, double(d.n_boundary) * (next.width + next.k) * es, 0)));
    }
    ctx->stats.fwd_elems[layer] += int64_t(d.n_halo) * rule.k;
    ctx->stats.full_fwd_elems[layer] += int64_t(d.n_halo) * fi;
    return VARCO_OK;
}

extern "C" int32_t varco_layer_bwd(varco_ctx* ctx, int32_t layer, int32_t q, const void* dx_out, const void* x_out,
                                   const void* x_local, const void* m_saved, const void* h1, const void* h0,
                                   void* dh1, void* dh0, void* dx_local, void* dz_halo, varco_stream stream) {
    if (ctx) ctx->prof.interrupt();   // events are shared between the launches of one call only
    if (int32_t rc = check_layer(ctx, layer, "varco_layer_bwd")) return rc;
    if (int32_t rc = check_part(ctx, q, "varco_layer_bwd")) return rc;
    const PartState& ps = ctx->parts[q];
    const varco_partition_desc& d = ps.d;
    const bool sage = ctx->conv == VARCO_CONV_SAGE;
    const bool transform_first = ctx->layers[layer].order == VARCO_ORDER_TRANSFORM_FIRST;
    if (!h1 || !dh1 || (d.n_local > 0 && (!dx_out || !x_out || !x_local || (!m_saved && !transform_first))))
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_layer_bwd: null pointer");
    if (sage && (!h0 || !dh0)) return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_layer_bwd: h0 and dh0 are required for the SAGE convolution");
    if (!sage && (h0 || dh0)) return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_layer_bwd: h0 and dh0 must be null for the single-tap convolution");
    if (!dx_local && dz_halo) return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_layer_bwd: dz_halo given without dx_local");
    if (dx_local && d.n_halo > 0 && !dz_halo && ctx->layers[layer].k > 0)
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_layer_bwd: dz_halo is null but the partition has halo nodes");
    if (int32_t rc = check_wide_rows(ctx, ctx->widths[layer], {dx_local, dz_halo}, "varco_layer_bwd")) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int32_t fi = ctx->widths[layer], fo = ctx->widths[layer + 1];
    const void* gate = ctx->act[layer] == VARCO_ACT_RELU ? x_out : nullptr;
    const int32_t nl = d.n_local;
    const int dt = ctx->dtype;
    const double es = ctx->elem_bytes();
    if (nl == 0) return VARCO_OK;
    Workspace* wsp = nullptr;
    if (int32_t rc = workspace_for(ctx, st, &wsp, "varco_layer_bwd")) return rc;
    Workspace& ws = *wsp;
    if (transform_first)
        return layer_bwd_transform_first(ctx, ps, ws, layer, dx_out, x_local, m_saved, h1, h0, dh1, dh0, dx_local, dz_halo, st);

    // weight gradients: reductions over the partition's rows, split over workgroups
    {
        GemmArgs g;
        g.m = fi, g.n = fo, g.k = nl;
        g.a.ptr = m_saved, g.a.ld = fi, g.a.transposed = true, g.a.dtype = dt;
        g.b.ptr = dx_out, g.b.gate = gate, g.b.ld = fo, g.b.dtype = dt;
        g.c = dh1, g.ldc = fo;
        g.accumulate = true;
        g.partial = ws.gemm;
        const LaunchTag wtag = ctx->tag(VARCO_K_GEMM_WGRAD, 0, 2.0 * fi * fo * double(nl));
        for (int tap = 0; tap < (sage ? 2 : 1); ++tap) {
            if (tap == 1) g.a.ptr = x_local, g.c = dh0;
            g.f32_terms = dt == VARCO_F32 ? ctx->f32_terms : 0;
            g.split_k = gemm_split_for(fi, fo, nl, gemm_kind(g));
            if (size_t(g.split_k) * fi * fo > ws.gemm_elems)
                return varco_fail(ctx, VARCO_ERR_STATE, "varco_layer_bwd: workspace too small");
            VARCO_HIP(ctx, varco_launch_gemm(g, st, wtag));
        }
    }
    if (!dx_local) return VARCO_OK;

    // dM = dZ H1^T
    {
        GemmArgs g;
        g.m = nl, g.n = fi, g.k = fo;
        g.a.ptr = dx_out, g.a.gate = gate, g.a.ld = fo, g.a.dtype = dt;
        g.b.ptr = h1, g.b.ld = fo, g.b.transposed = true;
        g.c = ws.dm, g.ldc = fi, g.c_dtype = dt;
        VARCO_HIP(ctx, prep_weight(ctx, ws, layer, h1, fi, fo, false, 0, false, st, g));
        VARCO_HIP(ctx, varco_launch_gemm(g, st, ctx->tag(VARCO_K_GEMM_DGRAD, 0, 2.0 * fi * fo * double(nl))));
    }
    // transposed aggregation: local rows in full, halo rows only at their kept positions
    const MaskRule rule = make_rule(ctx, layer);
    const MaskRule dense_rule = full_rule(fi);
    const double tl_bytes = double(ps.nnz_t_local) * 8.0 + (double(nl) + 1.0) * 4.0 + 2.0 * double(nl) * fi * es;
    const double th_out_bytes = (double(d.n_halo) + 1.0) * 4.0 + double(d.n_halo) * rule.k * es;
    const double th_bytes = double(d.nnz - ps.nnz_t_local) * 8.0 + double(nl) * fi * es + th_out_bytes;
    const double tl_stream = tl_bytes + (double(ps.nnz_t_local) - double(nl)) * fi * es;   // a source row per entry
    VARCO_HIP(ctx, varco_launch_spmm(dt, ps.t_local, nullptr, d.t_colidx, d.t_vals, ws.dm, nullptr, 0, dense_rule, dx_local,
                                     0, ws.spmm, st, ctx->tag(VARCO_K_AGG_BWD_LOCAL, tl_bytes, 0, tl_stream)));
    if (d.n_halo > 0 && rule.k > 0) {   // k = 0: nothing is handed back
        if (rule.k == rule.width) {
            VARCO_HIP(ctx, varco_launch_spmm(dt, ps.t_halo, nullptr, d.t_colidx, d.t_vals, ws.dm, nullptr, 0, dense_rule,
                                             dz_halo, nl, ws.spmm, st, ctx->tag(VARCO_K_AGG_BWD_HALO, th_bytes, 0)));
        } else {
            // product buffer: sized by varco_prepare / varco_set_ratio / varco_register_partition, never here
            const size_t need = (size_t(d.nnz - ps.nnz_t_local) * rule.k * size_t(es) + 3) / 4;   // in floats
            if (need > ws.prod_elems)
                return varco_fail(ctx, VARCO_ERR_STATE, "varco_layer_bwd: the stream's workspace is too small; call varco_prepare");
            VARCO_HIP(ctx, varco_launch_halo_grad(dt, ps.fwd, ps.t_halo, ps.edges, d.vals, ps.prow, int32_t(ps.nnz_t_local),
                                                  ws.dm, rule, ws.prod, dz_halo, nl, ws.spmm, st,
                                                  ctx->tag(VARCO_K_AGG_BWD_HALO, th_bytes - th_out_bytes, 0),
                                                  ctx->tag(VARCO_K_AGG_BWD_HALO_SUM, th_out_bytes, 0)));
        }
        ctx->stats.bwd_elems[layer] += int64_t(d.n_halo) * rule.k;
        ctx->stats.full_bwd_elems[layer] += int64_t(d.n_halo) * fi;
    }
    // self tap: dX_loc += dZ H0^T
    if (sage) {
        GemmArgs g;
        g.m = nl, g.n = fi, g.k = fo;
        g.a.ptr = dx_out, g.a.gate = gate, g.a.ld = fo, g.a.dtype = dt;
        g.b.ptr = h0, g.b.ld = fo, g.b.transposed = true;
        g.c = dx_local, g.ldc = fi, g.c_dtype = dt;
        g.accumulate = true;
        VARCO_HIP(ctx, prep_weight(ctx, ws, layer, h0, fi, fo, false, 1, false, st, g));
        VARCO_HIP(ctx, varco_launch_gemm(g, st, ctx->tag(VARCO_K_GEMM_DGRAD, 0, 2.0 * fi * fo * double(nl))));
    }
    return VARCO_OK;
}

// ---------------------------------------------------------------------------------------------------------
// Building blocks of a general K-tap layer: one hop of aggregation (forward / transposed) and the dense
// products, as separate calls.
// ---------------------------------------------------------------------------------------------------------

extern "C" int32_t varco_aggregate_fwd(varco_ctx* ctx, int32_t tap, int32_t q, const void* y_local, const void* z_in,
                                       void* y_out, varco_stream stream) {
    if (ctx) ctx->prof.interrupt();   // events are shared between the launches of one call only
    int32_t layer = tap, hop = 0;
    if (int32_t rc = split_tap(ctx, &layer, &hop, "varco_aggregate_fwd")) return rc;
    if (int32_t rc = check_part(ctx, q, "varco_aggregate_fwd")) return rc;
    const PartState& ps = ctx->parts[q];
    const varco_partition_desc& d = ps.d;
    if (d.n_local > 0 && (!y_local || !y_out)) return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_aggregate_fwd: null pointer");
    if (d.n_halo > 0 && !z_in && ctx->layers[layer].k > 0)
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_aggregate_fwd: z_in is null but the partition has halo nodes");
    if (int32_t rc = check_wide_rows(ctx, ctx->widths[layer], {y_local, z_in, y_out}, "varco_aggregate_fwd")) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    Workspace* wsp = nullptr;
    if (int32_t rc = workspace_for(ctx, st, &wsp, "varco_aggregate_fwd")) return rc;
    const int32_t fi = ctx->widths[layer];
    const MaskRule rule = make_rule(ctx, layer, hop);
    ctx->layers[layer].ran_forward = true;
    const double es = ctx->elem_bytes();
    const double bytes = double(d.nnz) * 8.0 + (double(d.n_local) + 1.0) * 4.0 + 2.0 * double(d.n_local) * fi * es +
                         double(d.n_halo) * rule.k * es;
    const double stream_bytes = double(d.nnz) * 8.0 + (double(d.n_local) + 1.0) * 4.0 + double(d.n_local) * fi * es +
                                double(ps.nnz_t_local) * fi * es + double(d.nnz - ps.nnz_t_local) * rule.k * es;
    VARCO_HIP(ctx, varco_launch_spmm(ctx->dtype, ps.fwd, ps.edges, nullptr, d.vals, y_local, z_in, ps.z_rows, rule, y_out, 0, wsp->spmm,
                                     st, ctx->tag(VARCO_K_AGG_FWD, bytes, 0, stream_bytes)));
    ctx->stats.fwd_elems[layer] += int64_t(d.n_halo) * rule.k;
    ctx->stats.full_fwd_elems[layer] += int64_t(d.n_halo) * fi;
    return VARCO_OK;
}

extern "C" int32_t varco_aggregate_bwd(varco_ctx* ctx, int32_t tap, int32_t q, const void* g_out, void* g_local,
                                       void* dz_halo, varco_stream stream) {
    if (ctx) ctx->prof.interrupt();   // events are shared between the launches of one call only
    int32_t layer = tap, hop = 0;
    if (int32_t rc = split_tap(ctx, &layer, &hop, "varco_aggregate_bwd")) return rc;
    if (int32_t rc = check_part(ctx, q, "varco_aggregate_bwd")) return rc;
    const PartState& ps = ctx->parts[q];
    const varco_partition_desc& d = ps.d;
    const int32_t nl = d.n_local;
    if (nl == 0) return VARCO_OK;
    if (!g_out || !g_local) return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_aggregate_bwd: null pointer");
    if (d.n_halo > 0 && !dz_halo && ctx->layers[layer].k > 0)
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_aggregate_bwd: dz_halo is null but the partition has halo nodes");
    if (int32_t rc = check_wide_rows(ctx, ctx->widths[layer], {g_out, g_local, dz_halo}, "varco_aggregate_bwd")) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    Workspace* wsp = nullptr;
    if (int32_t rc = workspace_for(ctx, st, &wsp, "varco_aggregate_bwd")) return rc;
    Workspace& ws = *wsp;
    const int dt = ctx->dtype;
    const double es = ctx->elem_bytes();
    const int32_t fi = ctx->widths[layer];
    const MaskRule rule = make_rule(ctx, layer, hop);
    const MaskRule dense_rule = full_rule(fi);
    const double tl_bytes = double(ps.nnz_t_local) * 8.0 + (double(nl) + 1.0) * 4.0 + 2.0 * double(nl) * fi * es;
    const double th_out_bytes = (double(d.n_halo) + 1.0) * 4.0 + double(d.n_halo) * rule.k * es;
    const double th_bytes = double(d.nnz - ps.nnz_t_local) * 8.0 + double(nl) * fi * es + th_out_bytes;
    const double tl_stream = tl_bytes + (double(ps.nnz_t_local) - double(nl)) * fi * es;
    VARCO_HIP(ctx, varco_launch_spmm(dt, ps.t_local, nullptr, d.t_colidx, d.t_vals, g_out, nullptr, 0, dense_rule, g_local, 0,
                                     ws.spmm, st, ctx->tag(VARCO_K_AGG_BWD_LOCAL, tl_bytes, 0, tl_stream)));
    if (d.n_halo > 0 && rule.k > 0) {
        if (rule.k == rule.width) {
            VARCO_HIP(ctx, varco_launch_spmm(dt, ps.t_halo, nullptr, d.t_colidx, d.t_vals, g_out, nullptr, 0, dense_rule, dz_halo,
                                             nl, ws.spmm, st, ctx->tag(VARCO_K_AGG_BWD_HALO, th_bytes, 0)));
        } else {
            const size_t need = (size_t(d.nnz - ps.nnz_t_local) * rule.k * size_t(es) + 3) / 4;   // in floats
            if (need > ws.prod_elems)
                return varco_fail(ctx, VARCO_ERR_STATE, "varco_aggregate_bwd: the stream's workspace is too small; call varco_prepare");
            VARCO_HIP(ctx, varco_launch_halo_grad(dt, ps.fwd, ps.t_halo, ps.edges, d.vals, ps.prow, int32_t(ps.nnz_t_local), g_out,
                                                  rule, ws.prod, dz_halo, nl, ws.spmm, st,
                                                  ctx->tag(VARCO_K_AGG_BWD_HALO, th_bytes - th_out_bytes, 0),
                                                  ctx->tag(VARCO_K_AGG_BWD_HALO_SUM, th_out_bytes, 0)));
        }
        ctx->stats.bwd_elems[layer] += int64_t(d.n_halo) * rule.k;
        ctx->stats.full_bwd_elems[layer] += int64_t(d.n_halo) * fi;
    }
    return VARCO_OK;
}

namespace {

// Shared checks of the dense-product calls; gate = x_out when the layer's activation is ReLU.
int32_t transform_prologue(varco_ctx* ctx, int32_t layer, int64_t n_rows, const char* fn) {
    if (int32_t rc = check_layer(ctx, layer, fn)) return rc;
    ctx->prof.interrupt();   // events are shared between the launches of one call only
    if (n_rows < 0 || n_rows >= (int64_t(1) << 31)) {
        std::string m = std::string(fn) + ": row count out of range";
        return varco_fail(ctx, VARCO_ERR_SHAPE, m.c_str());
    }
    return VARCO_OK;
}

}  // namespace

extern "C" int32_t varco_transform_fwd(varco_ctx* ctx, int32_t layer, int64_t n_rows, const void* y, const void* h, void* c,
                                       int32_t accumulate, int32_t apply_act, varco_stream stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    Workspace* ws = nullptr;
    if (int32_t rc = transform_prologue(ctx, layer, n_rows, "varco_transform_fwd")) return rc;
    if (n_rows == 0) return VARCO_OK;
    if (!y || !h || !c) return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_transform_fwd: null pointer");
    if (int32_t rc = workspace_for(ctx, st, &ws, "varco_transform_fwd")) return rc;
    const int32_t fi = ctx->widths[layer], fo = ctx->widths[layer + 1];
    const int dt = ctx->dtype;
    GemmArgs g;
    g.m = int32_t(n_rows), g.n = fo, g.k = fi;
    g.a.ptr = y, g.a.ld = fi, g.a.dtype = dt;
    g.b.ptr = h, g.b.ld = fo;
    g.c = c, g.ldc = fo, g.c_dtype = dt;
    g.accumulate = accumulate != 0;
    g.relu = apply_act != 0 && ctx->act[layer] == VARCO_ACT_RELU;
    VARCO_HIP(ctx, prep_weight(ctx, *ws, layer, h, fi, fo, true, 0, false, st, g));
    VARCO_HIP(ctx, varco_launch_gemm(g, st, ctx->tag(VARCO_K_GEMM_FWD, 0, 2.0 * double(g.m) * g.n * g.k)));
    return VARCO_OK;
}

extern "C" int32_t varco_transform_bwd_weight(varco_ctx* ctx, int32_t layer, int64_t n_rows, const void* y,
                                              const void* dx_out, const void* x_out, void* dh, varco_stream stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    Workspace* ws = nullptr;
    if (int32_t rc = transform_prologue(ctx, layer, n_rows, "varco_transform_bwd_weight")) return rc;
    if (n_rows == 0) return VARCO_OK;
    if (!y || !dx_out || !dh || (!x_out && ctx->act[layer] == VARCO_ACT_RELU))
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_transform_bwd_weight: null pointer");
    if (int32_t rc = workspace_for(ctx, st, &ws, "varco_transform_bwd_weight")) return rc;
    const int32_t fi = ctx->widths[layer], fo = ctx->widths[layer + 1];
    const int dt = ctx->dtype;
    GemmArgs g;
    g.m = fi, g.n = fo, g.k = int32_t(n_rows);
    g.a.ptr = y, g.a.ld = fi, g.a.transposed = true, g.a.dtype = dt;
    g.b.ptr = dx_out, g.b.gate = ctx->act[layer] == VARCO_ACT_RELU ? x_out : nullptr, g.b.ld = fo, g.b.dtype = dt;
    g.c = dh, g.ldc = fo;
    g.accumulate = true;
    g.partial = ws->gemm;
    g.f32_terms = dt == VARCO_F32 ? ctx->f32_terms : 0;
    g.split_k = gemm_split_for(fi, fo, n_rows, gemm_kind(g));
    if (size_t(g.split_k) * fi * fo > ws->gemm_elems) {   // rows beyond what the registered partitions sized
        const int64_t fit = int64_t(ws->gemm_elems / (size_t(fi) * fo));
        if (fit < 1) return varco_fail(ctx, VARCO_ERR_STATE, "varco_transform_bwd_weight: workspace too small (register a partition first)");
        g.split_k = int32_t(fit);
    }
    VARCO_HIP(ctx, varco_launch_gemm(g, st, ctx->tag(VARCO_K_GEMM_WGRAD, 0, 2.0 * fi * fo * double(n_rows))));
    return VARCO_OK;
}

extern "C" int32_t varco_transform_bwd_weight_static(varco_ctx* ctx, int32_t layer, int64_t n_rows, const void* y,
                                                     const void* dx_out, const void* x_out, void* dh, varco_stream stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (int32_t rc = transform_prologue(ctx, layer, n_rows, "varco_transform_bwd_weight_static")) return rc;
    if (n_rows == 0) return VARCO_OK;
    if (!y || !dx_out || !dh || (!x_out && ctx->act[layer] == VARCO_ACT_RELU))
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_transform_bwd_weight_static: null pointer");
    const int32_t fi = ctx->widths[layer], fo = ctx->widths[layer + 1];
    const int dt = ctx->dtype;
    GemmArgs g;
    g.m = fi, g.n = fo, g.k = int32_t(n_rows);
    g.a.ptr = y, g.a.ld = fi, g.a.transposed = true, g.a.dtype = dt;
    g.b.ptr = dx_out, g.b.gate = ctx->act[layer] == VARCO_ACT_RELU ? x_out : nullptr, g.b.ld = fo, g.b.dtype = dt;
    g.c = dh, g.ldc = fo;
    g.accumulate = true;
    g.f32_terms = dt == VARCO_F32 ? ctx->f32_terms : 0;
    g.split_k = gemm_split_for(fi, fo, n_rows, gemm_kind(g));
    const size_t need = g.split_k > 1 ? size_t(g.split_k) * fi * fo : 0;
    if (need > kScratchFloats) {
        char msg[256];
        std::snprintf(msg, sizeof msg,
                      "varco_transform_bwd_weight_static: %d x %d weights over %lld rows need %zu bytes of scratch, the static "
                      "array holds %zu; use varco_transform_bwd_weight", fi, fo, static_cast<long long>(n_rows),
                      need * sizeof(float), kScratchFloats * sizeof(float));
        return varco_fail(ctx, VARCO_ERR_SHAPE, msg);
    }
    float* ptr = nullptr;
    VARCO_HIP(ctx, scratch_of_current_device(&ptr));
    g.partial = ptr;   // every element of every slab the reduction reads is written first: nothing to clear
    VARCO_HIP(ctx, varco_launch_gemm(g, st, LaunchTag{}));   // not bracketed by profiler events (they would be created here)
    return VARCO_OK;
}

extern "C" int32_t varco_transform_bwd_input(varco_ctx* ctx, int32_t layer, int64_t n_rows, const void* dx_out,
                                             const void* x_out, const void* h, void* g_out, int32_t accumulate,
                                             varco_stream stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    Workspace* ws = nullptr;
    if (int32_t rc = transform_prologue(ctx, layer, n_rows, "varco_transform_bwd_input")) return rc;
    if (n_rows == 0) return VARCO_OK;
    if (!dx_out || !h || !g_out || (!x_out && ctx->act[layer] == VARCO_ACT_RELU))
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_transform_bwd_input: null pointer");
    if (int32_t rc = workspace_for(ctx, st, &ws, "varco_transform_bwd_input")) return rc;
    const int32_t fi = ctx->widths[layer], fo = ctx->widths[layer + 1];
    const int dt = ctx->dtype;
    GemmArgs g;
    g.m = int32_t(n_rows), g.n = fi, g.k = fo;
    g.a.ptr = dx_out, g.a.gate = ctx->act[layer] == VARCO_ACT_RELU ? x_out : nullptr, g.a.ld = fo, g.a.dtype = dt;
    g.b.ptr = h, g.b.ld = fo, g.b.transposed = true;
    g.c = g_out, g.ldc = fi, g.c_dtype = dt;
    g.accumulate = accumulate != 0;
    VARCO_HIP(ctx, prep_weight(ctx, *ws, layer, h, fi, fo, false, 0, false, st, g));
    VARCO_HIP(ctx, varco_launch_gemm(g, st, ctx->tag(VARCO_K_GEMM_DGRAD, 0, 2.0 * fi * fo * double(n_rows))));
    return VARCO_OK;
}

extern "C" int32_t varco_accumulate_returned(varco_ctx* ctx, int32_t layer, int32_t p, const int32_t* ret_ptr,
                                             const int32_t* ret_src, const void* returned, void* dx_local,
                                             varco_stream stream) {
    if (ctx) ctx->prof.interrupt();   // events are shared between the launches of one call only
    int32_t hop = 0;
    if (int32_t rc = split_tap(ctx, &layer, &hop, "varco_accumulate_returned")) return rc;
    if (int32_t rc = check_part(ctx, p, "varco_accumulate_returned")) return rc;
    const PartState& ps = ctx->parts[p];
    if (ps.d.n_boundary == 0 || ctx->layers[layer].k == 0) return VARCO_OK;
    if ((ret_ptr == nullptr) != (ret_src == nullptr))
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_accumulate_returned: ret_ptr and ret_src go together");
    if (!ret_ptr) {
        if (!ps.d.ret_ptr) return varco_fail(ctx, VARCO_ERR_STATE, "varco_accumulate_returned: no map was given at registration");
        ret_ptr = ps.d.ret_ptr, ret_src = ps.d.ret_src;
    }
    if (!returned || !dx_local) return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_accumulate_returned: null pointer");
    ctx->layers[layer].ran_forward = true;
    const MaskRule rule = make_rule(ctx, layer, hop);
    // the map's two index arrays, every returned row once, and the owner-side read-modify-write of k values per
    // boundary row (the number of returned rows is known for the registered map only)
    const double n_ret = ret_ptr == ps.d.ret_ptr ? double(ps.n_returned) : 0.0;
    const double bytes = (double(ps.d.n_boundary) + 1.0 + n_ret) * 4.0 +
                         (n_ret + 2.0 * double(ps.d.n_boundary)) * rule.k * ctx->elem_bytes();
    VARCO_HIP(ctx, varco_launch_accumulate_returned(ctx->dtype, rule, ps.boundary_gid, ps.d.boundary_rows, ps.d.n_boundary,
                                                    ret_ptr, ret_src, returned, dx_local, ctx->widths[layer],
                                                    static_cast<hipStream_t>(stream), ctx->tag(VARCO_K_DECOMPRESS, bytes, 0)));
    return VARCO_OK;
}

extern "C" int32_t varco_get_stats(const varco_ctx* ctx, varco_stats* out) {
    if (!ctx) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_get_stats: null context");
    if (!out) return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_get_stats: null output");
    *out = ctx->stats;
    return VARCO_OK;
}

extern "C" int32_t varco_reset_stats(varco_ctx* ctx) {
    if (!ctx) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_reset_stats: null context");
    const int32_t b = ctx->stats.bytes_per_elem;
    ctx->stats = varco_stats{};
    ctx->stats.bytes_per_elem = b;
    return VARCO_OK;
}

extern "C" int32_t varco_softmax_xent(varco_ctx* ctx, const void* logits, int64_t ld, const int32_t* labels, int64_t n_rows,
                                      int32_t n_classes, float scale, void* dlogits, int64_t ldd, float* row_loss,
                                      int32_t* row_correct, float* totals, varco_stream stream) {
    if (!ctx) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_softmax_xent: null context");
    if (n_rows < 0 || n_classes < 1 || n_classes > VARCO_MAX_WIDTH)
        return varco_fail(ctx, VARCO_ERR_SHAPE, "varco_softmax_xent: row count or class count out of range");
    if (ld < n_classes || (dlogits && ldd < n_classes))
        return varco_fail(ctx, VARCO_ERR_SHAPE, "varco_softmax_xent: leading dimension smaller than the class count");
    if (n_rows == 0) return VARCO_OK;
    if (!logits || !labels || !row_loss || !row_correct)
        return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_softmax_xent: null pointer");
    VARCO_HIP(ctx, varco_launch_softmax_xent(ctx->dtype, logits, ld, labels, n_rows, n_classes, scale, dlogits, ldd, row_loss,
                                             row_correct, totals, static_cast<hipStream_t>(stream)));
    return VARCO_OK;
}

extern "C" int32_t varco_sgd_step(void* w, const void* dw, int64_t n, float lr, varco_stream stream) {
    if (n < 0) return varco_fail(nullptr, VARCO_ERR_SHAPE, "varco_sgd_step: negative count");
    if (n == 0) return VARCO_OK;
    if (!w || !dw) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_sgd_step: null pointer");
    VARCO_HIP(static_cast<const varco_ctx*>(nullptr),
              varco_launch_sgd(static_cast<float*>(w), static_cast<const float*>(dw), n, lr, static_cast<hipStream_t>(stream)));
    return VARCO_OK;
}

extern "C" int32_t varco_schedule_ratio(int32_t kind, int64_t step, int64_t n_steps, uint32_t c_max, uint32_t c_min,
                                        uint32_t param, uint32_t* num, uint32_t* den) {
    if (!num || !den) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_schedule_ratio: null output");
    if (c_min < 1 || c_max < c_min || n_steps < 1 || step < 0)
        return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_schedule_ratio: need 1 <= c_min <= c_max, n_steps >= 1, step >= 0");
    uint64_t n = c_min, d = 1;
    if (kind == VARCO_SCHED_LINEAR) {
        // c_max - slope (c_max - c_min) step / K over the common denominator K, in 128-bit integers
        const __int128 top = __int128(c_max) * n_steps - __int128(param) * (c_max - c_min) * step;
        if (top > __int128(c_min) * n_steps) {
            if (top > __int128(0xFFFFFFFFu) || n_steps > int64_t(0xFFFFFFFFu))
                return varco_fail(nullptr, VARCO_ERR_SHAPE, "varco_schedule_ratio: ratio does not fit 32-bit integers");
            const uint64_t g = std::gcd(uint64_t(top), uint64_t(n_steps));
            n = uint64_t(top) / g, d = uint64_t(n_steps) / g;
        }
    } else if (kind == VARCO_SCHED_FIXED_INCREMENT) {
        const __int128 v = __int128(c_max) - __int128(param) * step;
        n = v > __int128(c_min) ? uint64_t(v) : c_min;
    } else if (kind == VARCO_SCHED_EXPONENTIAL) {
        if (param < 2) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_schedule_ratio: the base must be an integer >= 2");
        const int64_t exponent = std::max<int64_t>(n_steps - step + 1, 0);
        uint64_t value = 1;
        bool capped = false;
        for (int64_t i = 0; i < exponent && !capped; ++i) {
            value *= param;              // value < c_max <= 2^32 before the product: no overflow in 64 bits
            capped = value >= c_max;
        }
        n = capped ? c_max : std::max<uint64_t>(value, c_min);
    } else {
        return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_schedule_ratio: unknown schedule");
    }
    *num = uint32_t(n), *den = uint32_t(d);
    return VARCO_OK;
}

extern "C" int32_t varco_sum_gradients(void* dst, const void* src, int64_t n, varco_stream stream) {
    if (n < 0) return varco_fail(nullptr, VARCO_ERR_SHAPE, "varco_sum_gradients: negative count");
    if (n == 0) return VARCO_OK;
    if (!dst || !src) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_sum_gradients: null pointer");
    VARCO_HIP(static_cast<const varco_ctx*>(nullptr),
              varco_launch_sum_gradients(static_cast<float*>(dst), static_cast<const float*>(src), n,
                                         static_cast<hipStream_t>(stream)));
    return VARCO_OK;
}

extern "C" int32_t varco_calibration_copy(void* dst, const void* src, int64_t bytes, varco_stream stream) {
    if (bytes < 0 || bytes % 16 != 0) return varco_fail(nullptr, VARCO_ERR_SHAPE, "varco_calibration_copy: bytes must be a non-negative multiple of 16");
    if (bytes == 0) return VARCO_OK;
    if (!dst || !src || (reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) % 16 != 0)
        return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_calibration_copy: null or misaligned pointer");
    VARCO_HIP(static_cast<const varco_ctx*>(nullptr),
              varco_launch_calibration_copy(dst, src, bytes, static_cast<hipStream_t>(stream)));
    return VARCO_OK;
}

extern "C" int32_t varco_profile_enable(varco_ctx* ctx, int32_t on) {
    if (!ctx) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_profile_enable: null context");
    ctx->prof.on = on != 0;
    return VARCO_OK;
}

extern "C" int32_t varco_profile_read(varco_ctx* ctx, varco_profile* out, int32_t reset) {
    if (!ctx) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_profile_read: null context");
    if (!out) return varco_fail(ctx, VARCO_ERR_INVALID_ARG, "varco_profile_read: null output");
    for (VarcoProfiler::Rec& r : ctx->prof.recs) {
        if (r.stop < 0) continue;
        VARCO_HIP(ctx, hipEventSynchronize(ctx->prof.events[r.stop]));
        float ms = 0.f;
        VARCO_HIP(ctx, hipEventElapsedTime(&ms, ctx->prof.events[r.start], ctx->prof.events[r.stop]));
        ctx->prof_ms[r.cls] += ms;
        ctx->prof_bytes[r.cls] += r.bytes;
        ctx->prof_stream_bytes[r.cls] += r.stream_bytes;
        ctx->prof_flops[r.cls] += r.flops;
        ctx->prof_launches[r.cls] += 1;
    }
    for (hipEvent_t e : ctx->prof.events) ctx->prof.pool.push_back(e);
    ctx->prof.events.clear();
    ctx->prof.last_stop = -1;
    ctx->prof.recs.clear();
    for (int c = 0; c < VARCO_K_COUNT; ++c) {
        out->launches[c] = ctx->prof_launches[c];
        out->ms[c] = ctx->prof_ms[c];
        out->bytes[c] = ctx->prof_bytes[c];
        out->flops[c] = ctx->prof_flops[c];
        out->stream_bytes[c] = ctx->prof_stream_bytes[c];
        if (reset) ctx->prof_launches[c] = 0, ctx->prof_ms[c] = ctx->prof_bytes[c] = ctx->prof_flops[c] = ctx->prof_stream_bytes[c] = 0.0;
    }
    return VARCO_OK;
}
