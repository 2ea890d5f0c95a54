// Host-side construction of every partition's index structures from a global CSR operator and a
// node -> partition map (Section III of the paper: local nodes, remote neighbours, boundary nodes).
// Counting-sort based, O(nnz + n) per partition plus a sort of each partition's halo list; partitions
// are built concurrently on host threads. The orderings produced here are the library's contract:
// local ids ascending by global id, halo slots by (owner, global id), columns ascending within a row
// (local columns first), transpose rows ascending by local row.
#include <algorithm>
#include <atomic>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <string>
#include <thread>
#include <vector>

#include "varco_internal.h"

struct HostPart {
    int32_t n_local = 0, n_halo = 0, n_boundary = 0, z_row_offset = 0, halo_row_offset = 0;
    int64_t nnz = 0;
    std::vector<int32_t> rowptr, colidx, t_rowptr, t_colidx, local_gid, halo_gid, halo_owner_ptr,
        boundary_rows, halo_src_row, halo_zrow, ret_ptr, ret_src;
    std::vector<float> vals, t_vals;
};

struct varco_host_parts {
    int32_t n = 0, n_parts = 0;
    std::vector<HostPart> parts;
};

namespace {

struct SlotVal {
    int32_t col;
    float val;
};

// Builds everything of partition q that does not depend on other partitions' boundary lists.
void build_one(int32_t q, int32_t n, const int64_t* rowptr, const int32_t* colidx, const float* vals,
               const int32_t* part, const int32_t* local_index, int32_t n_parts, HostPart& hp,
               std::vector<int32_t>& slot_of /* size n, scratch, any content */, std::string& err) {
    const int32_t n_local = hp.n_local;
    // pass 1: entry count and the distinct remote columns
    int64_t nnz = 0;
    std::vector<uint64_t> halo_keys;
    for (int32_t i = 0; i < n_local; ++i) {
        const int32_t v = hp.local_gid[i];
        nnz += rowptr[v + 1] - rowptr[v];
    }
    if (nnz >= (int64_t(1) << 31)) {
        err = "partition " + std::to_string(q) + " has 2^31 or more entries";
        return;
    }
    // mark remote columns; slot_of[c] = -2 means "seen in this partition"
    for (int32_t i = 0; i < n_local; ++i) {
        const int32_t v = hp.local_gid[i];
        for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
            const int32_t c = colidx[e];
            if (part[c] != q && slot_of[c] != -2) {
                slot_of[c] = -2;
                halo_keys.push_back((uint64_t(uint32_t(part[c])) << 32) | uint32_t(c));
            }
        }
    }
    std::sort(halo_keys.begin(), halo_keys.end());
    const int32_t n_halo = int32_t(halo_keys.size());
    hp.n_halo = n_halo;
    hp.nnz = nnz;
    hp.halo_gid.resize(n_halo);
    hp.halo_owner_ptr.assign(n_parts + 1, 0);
    for (int32_t s = 0; s < n_halo; ++s) {
        const int32_t c = int32_t(halo_keys[s] & 0xFFFFFFFFu);
        hp.halo_gid[s] = c;
        slot_of[c] = s;
        hp.halo_owner_ptr[int32_t(halo_keys[s] >> 32) + 1]++;
    }
    for (int32_t p = 0; p < n_parts; ++p) hp.halo_owner_ptr[p + 1] += hp.halo_owner_ptr[p];

    // pass 2: renumbered row block; local columns keep their order, remote ones are sorted by slot
    hp.rowptr.resize(size_t(n_local) + 1);
    hp.colidx.resize(size_t(nnz));
    hp.vals.resize(size_t(nnz));
    std::vector<int32_t> t_count(size_t(n_local) + n_halo + 1, 0);
    std::vector<SlotVal> remote;
    int64_t w = 0;
    for (int32_t i = 0; i < n_local; ++i) {
        hp.rowptr[i] = int32_t(w);
        const int32_t v = hp.local_gid[i];
        remote.clear();
        int32_t prev = -1;
        for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
            const int32_t c = colidx[e];
            if (c <= prev) {
                err = "columns of row " + std::to_string(v) + " are not strictly ascending";
                return;
            }
            prev = c;
            if (part[c] == q) {
                hp.colidx[w] = local_index[c];
                hp.vals[w] = vals[e];
                ++w;
            } else {
                remote.push_back({n_local + slot_of[c], vals[e]});
            }
        }
        std::sort(remote.begin(), remote.end(), [](const SlotVal& a, const SlotVal& b) { return a.col < b.col; });
        for (const SlotVal& sv : remote) {
            hp.colidx[w] = sv.col;
            hp.vals[w] = sv.val;
            ++w;
        }
    }
    hp.rowptr[n_local] = int32_t(w);
    for (int64_t e = 0; e < nnz; ++e) t_count[size_t(hp.colidx[e]) + 1]++;

    // transpose by counting sort on the column; rows are visited in ascending order
    hp.t_rowptr.resize(size_t(n_local) + n_halo + 1);
    hp.t_rowptr[0] = 0;
    for (size_t c = 0; c < size_t(n_local) + n_halo; ++c) hp.t_rowptr[c + 1] = hp.t_rowptr[c] + t_count[c + 1];
    std::vector<int32_t> cursor(hp.t_rowptr.begin(), hp.t_rowptr.end() - 1);
    hp.t_colidx.resize(size_t(nnz));
    hp.t_vals.resize(size_t(nnz));
    for (int32_t i = 0; i < n_local; ++i) {
        for (int32_t e = hp.rowptr[i]; e < hp.rowptr[i + 1]; ++e) {
            const int32_t pos = cursor[hp.colidx[e]]++;
            hp.t_colidx[pos] = i;
            hp.t_vals[pos] = hp.vals[e];
        }
    }
    // leave slot_of clean of this partition's sentinel values is unnecessary: every later use first
    // overwrites the entries it reads (marks are only tested against -2 after being set by the same q)
    for (int32_t s = 0; s < n_halo; ++s) slot_of[hp.halo_gid[s]] = -1;
}

}  // namespace

extern "C" int32_t varco_partition_build(int32_t n, const int64_t* rowptr, const int32_t* colidx,
                                         const float* vals, const int32_t* part, int32_t n_parts,
                                         varco_host_parts** out) {
    if (!out) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_partition_build: out is null");
    *out = nullptr;
    if (!rowptr || !colidx || !vals || !part)
        return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_partition_build: null input array");
    if (n < 1 || n_parts < 1) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_partition_build: n and n_parts must be positive");
    if (rowptr[0] != 0) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_partition_build: rowptr[0] must be 0");
    for (int32_t v = 0; v < n; ++v) {
        if (part[v] < 0 || part[v] >= n_parts)
            return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_partition_build: part[v] outside [0, n_parts)");
        if (rowptr[v + 1] < rowptr[v])
            return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_partition_build: rowptr is not non-decreasing");
    }
    const int64_t nnz = rowptr[n];
    for (int64_t e = 0; e < nnz; ++e)
        if (colidx[e] < 0 || colidx[e] >= n)
            return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_partition_build: column index outside [0, n)");

    auto* h = new varco_host_parts;
    h->n = n;
    h->n_parts = n_parts;
    h->parts.resize(n_parts);
    std::vector<int32_t> local_index(n);
    for (int32_t v = 0; v < n; ++v) {
        HostPart& hp = h->parts[part[v]];
        local_index[v] = hp.n_local++;
        hp.local_gid.push_back(v);
    }

    // partitions in parallel; each worker owns one scratch map of n entries
    unsigned hw = std::thread::hardware_concurrency();
    int n_workers = int(std::min<unsigned>(std::min<unsigned>(hw ? hw : 4, 16), unsigned(n_parts)));
    std::vector<std::string> errors(n_parts);
    std::atomic<int32_t> next(0);
    auto worker = [&]() {
        std::vector<int32_t> slot_of(size_t(n), -1);
        for (;;) {
            const int32_t q = next.fetch_add(1);
            if (q >= n_parts) break;
            build_one(q, n, rowptr, colidx, vals, part, local_index.data(), n_parts, h->parts[q], slot_of,
                      errors[q]);
        }
    };
    std::vector<std::thread> pool;
    for (int t = 1; t < n_workers; ++t) pool.emplace_back(worker);
    worker();
    for (auto& t : pool) t.join();
    for (int32_t q = 0; q < n_parts; ++q) {
        if (!errors[q].empty()) {
            const bool shape = errors[q].find("2^31") != std::string::npos;
            std::string msg = "varco_partition_build: " + errors[q];
            delete h;
            return varco_fail(nullptr, shape ? VARCO_ERR_SHAPE : VARCO_ERR_INVALID_ARG, msg.c_str());
        }
    }

    // boundary nodes: referenced by some other partition's halo
    std::vector<uint8_t> needed(size_t(n), 0);
    for (const HostPart& hp : h->parts)
        for (int32_t c : hp.halo_gid) needed[c] = 1;
    std::vector<int32_t> boundary_index(size_t(n), -1);
    std::vector<int32_t> offsets(n_parts);
    int64_t offset = 0;
    for (int32_t p = 0; p < n_parts; ++p) {
        HostPart& hp = h->parts[p];
        for (int32_t i = 0; i < hp.n_local; ++i) {
            if (needed[hp.local_gid[i]]) {
                boundary_index[hp.local_gid[i]] = int32_t(hp.boundary_rows.size());
                hp.boundary_rows.push_back(i);
            }
        }
        hp.n_boundary = int32_t(hp.boundary_rows.size());
        hp.z_row_offset = int32_t(offset);
        offsets[p] = int32_t(offset);
        offset += hp.n_boundary;
    }
    for (HostPart& hp : h->parts) {
        hp.halo_src_row.resize(hp.n_halo);
        hp.halo_zrow.resize(hp.n_halo);
        for (int32_t s = 0; s < hp.n_halo; ++s) {
            const int32_t c = hp.halo_gid[s];
            hp.halo_src_row[s] = boundary_index[c];
            hp.halo_zrow[s] = boundary_index[c] + offsets[part[c]];
        }
    }
    // owner side of the backward exchange: where the rows returned for each boundary row sit in the
    // concatenation of all consumers' halo rows. Consumers are visited in ascending order and a consumer holds
    // a node at most once, so each boundary row's list comes out ordered by consumer.
    int64_t halo_rows = 0;
    for (HostPart& hp : h->parts) {
        hp.halo_row_offset = int32_t(halo_rows);
        halo_rows += hp.n_halo;
        if (halo_rows >= (int64_t(1) << 31)) {
            delete h;
            return varco_fail(nullptr, VARCO_ERR_SHAPE, "varco_partition_build: 2^31 or more halo rows over all partitions");
        }
    }
    for (int32_t p = 0; p < n_parts; ++p) {
        HostPart& owner = h->parts[p];
        owner.ret_ptr.assign(size_t(owner.n_boundary) + 1, 0);
        for (const HostPart& hq : h->parts)
            for (int32_t s = hq.halo_owner_ptr[p]; s < hq.halo_owner_ptr[p + 1]; ++s) owner.ret_ptr[size_t(hq.halo_src_row[s]) + 1]++;
        for (int32_t b = 0; b < owner.n_boundary; ++b) owner.ret_ptr[b + 1] += owner.ret_ptr[b];
        owner.ret_src.resize(size_t(owner.ret_ptr[owner.n_boundary]));
        std::vector<int32_t> fill(owner.ret_ptr.begin(), owner.ret_ptr.end() - 1);
        for (const HostPart& hq : h->parts)
            for (int32_t s = hq.halo_owner_ptr[p]; s < hq.halo_owner_ptr[p + 1]; ++s)
                owner.ret_src[size_t(fill[hq.halo_src_row[s]]++)] = hq.halo_row_offset + s;
    }
    *out = h;
    return VARCO_OK;
}

extern "C" int32_t varco_partition_view(const varco_host_parts* h, int32_t q, varco_partition_desc* out) {
    if (!h || !out) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_partition_view: null argument");
    if (q < 0 || q >= h->n_parts) return varco_fail(nullptr, VARCO_ERR_INVALID_ARG, "varco_partition_view: q out of range");
    const HostPart& hp = h->parts[q];
    out->n_local = hp.n_local;
    out->n_halo = hp.n_halo;
    out->n_boundary = hp.n_boundary;
    out->z_row_offset = hp.z_row_offset;
    out->nnz = hp.nnz;
    out->halo_row_offset = hp.halo_row_offset;
    out->n_returned = int32_t(hp.ret_src.size());
    out->rowptr = hp.rowptr.data();
    out->colidx = hp.colidx.data();
    out->vals = hp.vals.data();
    out->t_rowptr = hp.t_rowptr.data();
    out->t_colidx = hp.t_colidx.data();
    out->t_vals = hp.t_vals.data();
    out->local_gid = hp.local_gid.data();
    out->halo_gid = hp.halo_gid.data();
    out->halo_owner_ptr = hp.halo_owner_ptr.data();
    out->boundary_rows = hp.boundary_rows.data();
    out->halo_src_row = hp.halo_src_row.data();
    out->halo_zrow = hp.halo_zrow.data();
    out->ret_ptr = hp.ret_ptr.data();
    out->ret_src = hp.ret_src.data();
    return VARCO_OK;
}

extern "C" void varco_partition_free(varco_host_parts* h) { delete h; }
