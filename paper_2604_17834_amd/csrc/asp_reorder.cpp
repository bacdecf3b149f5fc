// Host-side preprocessing of the paper's sparse-matrix evaluation (Section IV-A, "Baselines and datasets"):
// Reverse Cuthill-McKee reordering of a square matrix's structure, permutation of CSR arrays, and a reader for
// Matrix Market coordinate files.  No GPU call anywhere in this file.
#include <algorithm>
#include <cctype>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <numeric>

#include "asp_internal.h"

struct asp_mtx {
    int64_t m = 0, k = 0;
    std::vector<int32_t> row_ptr, col_idx;
    std::vector<float> values;
};

namespace asp {
namespace {

// Neighbour lists of the structure of A + A^T, each sorted and free of duplicates (a stored diagonal entry makes
// a node its own neighbour, which only adds one to its degree).
void symmetric_structure(int64_t m, const int32_t *row_ptr, const int32_t *col_idx, std::vector<int64_t> &ptr,
                         std::vector<int32_t> &adj) {
    std::vector<int64_t> cnt(m + 1, 0);
    for (int64_t i = 0; i < m; ++i)
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
            ++cnt[i + 1];
            if (col_idx[p] != i) ++cnt[col_idx[p] + 1];
        }
    for (int64_t i = 0; i < m; ++i) cnt[i + 1] += cnt[i];
    std::vector<int32_t> raw(cnt[m]);
    std::vector<int64_t> fill(cnt.begin(), cnt.end() - 1);
    for (int64_t i = 0; i < m; ++i)
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
            const int32_t j = col_idx[p];
            raw[fill[i]++] = j;
            if (j != i) raw[fill[j]++] = (int32_t)i;
        }
    ptr.assign(m + 1, 0);
    adj.clear();
    adj.reserve(raw.size());
    for (int64_t i = 0; i < m; ++i) {
        std::sort(raw.begin() + cnt[i], raw.begin() + cnt[i + 1]);
        auto last = std::unique(raw.begin() + cnt[i], raw.begin() + cnt[i + 1]);
        adj.insert(adj.end(), raw.begin() + cnt[i], last);
        ptr[i + 1] = (int64_t)adj.size();
    }
}

bool is_permutation(const int32_t *p, int64_t n) {
    std::vector<uint8_t> seen(n, 0);
    for (int64_t i = 0; i < n; ++i) {
        if (p[i] < 0 || p[i] >= n || seen[p[i]]) return false;
        seen[p[i]] = 1;
    }
    return true;
}

std::string lower(std::string s) {
    for (auto &c : s) c = (char)std::tolower((unsigned char)c);
    return s;
}

}  // namespace
}  // namespace asp

using namespace asp;

extern "C" {

asp_status_t asp_rcm(int64_t m, const int32_t *row_ptr, const int32_t *col_idx, int32_t *perm) {
    if (!row_ptr || !perm) return fail(ASP_ERR_INVALID_ARG, "null row_ptr or perm");
    if (m < 1 || m >= (1ll << 31)) return fail(ASP_ERR_INVALID_ARG, "m out of range");
    if (row_ptr[m] > 0 && !col_idx) return fail(ASP_ERR_INVALID_ARG, "null col_idx");
    std::string why = validate_csr(m, m, row_ptr[m], row_ptr, col_idx);
    if (!why.empty()) return fail(ASP_ERR_INVALID_CSR, why);
    try {
        std::vector<int64_t> ptr;
        std::vector<int32_t> adj;
        symmetric_structure(m, row_ptr, col_idx, ptr, adj);
        // degree of a node = its neighbours in A + A^T, a stored diagonal entry counting twice (the convention of
        // the routine the paper names, so that both order neighbours by the same key)
        std::vector<int32_t> deg(m);
        for (int64_t v = 0; v < m; ++v) {
            deg[v] = (int32_t)(ptr[v + 1] - ptr[v]);
            if (std::binary_search(adj.begin() + ptr[v], adj.begin() + ptr[v + 1], (int32_t)v)) ++deg[v];
        }
        auto degree = [&](int32_t v) { return deg[v]; };
        auto lighter = [&](int32_t a, int32_t b) { return degree(a) != degree(b) ? degree(a) < degree(b) : a < b; };
        // start nodes in order of degree: every component begins at its unvisited node of least degree
        std::vector<int32_t> by_degree(m);
        std::iota(by_degree.begin(), by_degree.end(), 0);
        std::sort(by_degree.begin(), by_degree.end(), lighter);
        std::vector<uint8_t> visited(m, 0);
        std::vector<int32_t> order;
        order.reserve(m);
        size_t head = 0;
        for (int64_t s = 0; s < m; ++s) {
            if (visited[by_degree[s]]) continue;
            visited[by_degree[s]] = 1;
            order.push_back(by_degree[s]);
            // breadth-first: the not-yet-numbered neighbours of each node follow as one run, lightest first
            for (; head < order.size(); ++head) {
                const int32_t v = order[head];
                const size_t first = order.size();
                for (int64_t p = ptr[v]; p < ptr[v + 1]; ++p)
                    if (!visited[adj[p]]) {
                        visited[adj[p]] = 1;
                        order.push_back(adj[p]);
                    }
                std::sort(order.begin() + first, order.end(), lighter);
            }
        }
        for (int64_t i = 0; i < m; ++i) perm[i] = order[m - 1 - i];  // the reverse numbering
    } catch (const std::bad_alloc &) {
        return fail(ASP_ERR_OUT_OF_MEMORY, "host allocation failed in asp_rcm");
    }
    return ASP_OK;
}

asp_status_t asp_permute_csr(int64_t m, int64_t k, const int32_t *row_ptr, const int32_t *col_idx, const void *values,
                             int32_t dtype, const int32_t *row_perm, const int32_t *col_perm, int32_t *out_row_ptr,
                             int32_t *out_col_idx, void *out_values) {
    if (!row_ptr || !row_perm || !out_row_ptr) return fail(ASP_ERR_INVALID_ARG, "null row_ptr, row_perm or out_row_ptr");
    if (m < 1 || k < 1 || m >= (1ll << 31) || k >= (1ll << 31)) return fail(ASP_ERR_INVALID_ARG, "m or k out of range");
    if (dtype != ASP_DT_BF16 && dtype != ASP_DT_F32) return fail(ASP_ERR_INVALID_ARG, "unknown dtype");
    const int64_t nnz = row_ptr[m];
    if (nnz > 0 && (!col_idx || !values || !out_col_idx || !out_values))
        return fail(ASP_ERR_INVALID_ARG, "null column or value array with nnz > 0");
    std::string why = validate_csr(m, k, nnz, row_ptr, col_idx);
    if (!why.empty()) return fail(ASP_ERR_INVALID_CSR, why);
    if (!is_permutation(row_perm, m)) return fail(ASP_ERR_INVALID_ARG, "row_perm is not a permutation of 0..m-1");
    if (col_perm && !is_permutation(col_perm, k)) return fail(ASP_ERR_INVALID_ARG, "col_perm is not a permutation of 0..k-1");
    try {
        const size_t es = dtype_size(dtype);
        std::vector<int32_t> new_col_of;
        if (col_perm) {
            new_col_of.resize(k);
            for (int64_t j = 0; j < k; ++j) new_col_of[col_perm[j]] = (int32_t)j;
        }
        out_row_ptr[0] = 0;
        std::vector<std::pair<int32_t, int64_t>> row;  // (new column, position of the entry in the input)
        for (int64_t i = 0; i < m; ++i) {
            const int64_t old = row_perm[i];
            row.clear();
            for (int64_t p = row_ptr[old]; p < row_ptr[old + 1]; ++p)
                row.emplace_back(col_perm ? new_col_of[col_idx[p]] : col_idx[p], p);
            if (col_perm) std::sort(row.begin(), row.end());
            int64_t q = out_row_ptr[i];
            for (const auto &e : row) {
                out_col_idx[q] = e.first;
                std::memcpy((uint8_t *)out_values + (size_t)q * es, (const uint8_t *)values + (size_t)e.second * es, es);
                ++q;
            }
            out_row_ptr[i + 1] = (int32_t)q;
        }
    } catch (const std::bad_alloc &) {
        return fail(ASP_ERR_OUT_OF_MEMORY, "host allocation failed in asp_permute_csr");
    }
    return ASP_OK;
}

asp_status_t asp_mtx_read(const char *path, asp_mtx_t **out) {
    if (out) *out = nullptr;
    if (!path || !out) return fail(ASP_ERR_INVALID_ARG, "null path or out");
    FILE *f = std::fopen(path, "r");
    if (!f) return fail(ASP_ERR_INVALID_ARG, std::string("cannot open ") + path);
    struct Closer {
        FILE *f;
        ~Closer() { std::fclose(f); }
    } closer{f};
    try {
        std::vector<char> line(1 << 16);
        if (!std::fgets(line.data(), (int)line.size(), f)) return fail(ASP_ERR_INVALID_CSR, "empty file");
        char banner[64], object[64], format[64], field[64], symmetry[64];
        if (std::sscanf(line.data(), "%63s %63s %63s %63s %63s", banner, object, format, field, symmetry) != 5 ||
            lower(banner) != "%%matrixmarket" || lower(object) != "matrix")
            return fail(ASP_ERR_INVALID_CSR, "not a Matrix Market matrix header");
        const std::string fmt = lower(format), fld = lower(field), sym = lower(symmetry);
        if (fmt != "coordinate") return fail(ASP_ERR_UNSUPPORTED, "only coordinate (sparse) files are read");
        if (fld != "real" && fld != "integer" && fld != "pattern" && fld != "double")
            return fail(ASP_ERR_UNSUPPORTED, "field '" + fld + "' is not read (real, integer and pattern are)");
        if (sym != "general" && sym != "symmetric" && sym != "skew-symmetric")
            return fail(ASP_ERR_UNSUPPORTED, "symmetry '" + sym + "' is not read");
        const bool pattern = fld == "pattern";
        long long rows = 0, cols = 0, entries = 0;
        for (;;) {  // comments and blank lines, then the size line
            if (!std::fgets(line.data(), (int)line.size(), f)) return fail(ASP_ERR_INVALID_CSR, "no size line");
            const char *s = line.data();
            while (*s == ' ' || *s == '\t') ++s;
            if (*s == '%' || *s == '\n' || *s == '\r' || *s == 0) continue;
            if (std::sscanf(s, "%lld %lld %lld", &rows, &cols, &entries) != 3)
                return fail(ASP_ERR_INVALID_CSR, "malformed size line");
            break;
        }
        if (rows < 1 || cols < 1 || entries < 0 || rows >= (1ll << 31) || cols >= (1ll << 31) || entries >= (1ll << 30))
            return fail(ASP_ERR_UNSUPPORTED, "sizes out of range");
        struct Entry {
            int32_t r, c;
            double v;
        };
        std::vector<Entry> e;
        e.reserve((size_t)entries * (sym == "general" ? 1 : 2));
        for (long long n = 0; n < entries;) {
            if (!std::fgets(line.data(), (int)line.size(), f))
                return fail(ASP_ERR_INVALID_CSR, "file ends after " + std::to_string(n) + " of " + std::to_string(entries) + " entries");
            char *s = line.data();
            while (*s == ' ' || *s == '\t') ++s;
            if (*s == '%' || *s == '\n' || *s == '\r' || *s == 0) continue;
            char *end = nullptr;
            const long long r = std::strtoll(s, &end, 10);
            if (end == s) return fail(ASP_ERR_INVALID_CSR, "malformed entry line " + std::to_string(n + 1));
            s = end;
            const long long c = std::strtoll(s, &end, 10);
            if (end == s) return fail(ASP_ERR_INVALID_CSR, "malformed entry line " + std::to_string(n + 1));
            s = end;
            double v = 1.0;
            if (!pattern) {
                v = std::strtod(s, &end);
                if (end == s) return fail(ASP_ERR_INVALID_CSR, "entry line " + std::to_string(n + 1) + " has no value");
            }
            if (r < 1 || r > rows || c < 1 || c > cols)
                return fail(ASP_ERR_INVALID_CSR, "entry " + std::to_string(n + 1) + " lies outside the matrix");
            e.push_back({(int32_t)(r - 1), (int32_t)(c - 1), v});
            if (sym != "general" && r != c) e.push_back({(int32_t)(c - 1), (int32_t)(r - 1), sym == "symmetric" ? v : -v});
            ++n;
        }
        std::stable_sort(e.begin(), e.end(), [](const Entry &a, const Entry &b) { return a.r != b.r ? a.r < b.r : a.c < b.c; });
        asp_mtx *mx = new asp_mtx();
        mx->m = rows;
        mx->k = cols;
        mx->row_ptr.assign(rows + 1, 0);
        for (size_t i = 0; i < e.size();) {  // equal positions are summed in fp64, explicit zeros stay stored
            size_t j = i;
            double sum = 0.0;
            while (j < e.size() && e[j].r == e[i].r && e[j].c == e[i].c) sum += e[j++].v;
            mx->col_idx.push_back(e[i].c);
            mx->values.push_back((float)sum);
            ++mx->row_ptr[e[i].r + 1];
            i = j;
        }
        for (long long i = 0; i < rows; ++i) mx->row_ptr[i + 1] += mx->row_ptr[i];
        *out = mx;
    } catch (const std::bad_alloc &) {
        return fail(ASP_ERR_OUT_OF_MEMORY, "host allocation failed while reading the file");
    }
    return ASP_OK;
}

asp_status_t asp_mtx_get(const asp_mtx_t *mx, int64_t *m, int64_t *k, int64_t *nnz, const int32_t **row_ptr,
                         const int32_t **col_idx, const float **values) {
    if (!mx) return fail(ASP_ERR_INVALID_ARG, "null matrix");
    if (m) *m = mx->m;
    if (k) *k = mx->k;
    if (nnz) *nnz = (int64_t)mx->col_idx.size();
    if (row_ptr) *row_ptr = mx->row_ptr.data();
    if (col_idx) *col_idx = mx->col_idx.data();
    if (values) *values = mx->values.data();
    return ASP_OK;
}

asp_status_t asp_mtx_free(asp_mtx_t *mx) {
    delete mx;
    return ASP_OK;
}

}  // extern "C"
