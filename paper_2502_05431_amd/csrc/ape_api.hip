// Host side of the C ABI declared in include/ape.h: argument validation, split planning,
// workspace carving and kernel launches.  Nothing here allocates, copies or synchronises.
#include "ape_internal.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <initializer_list>
#include <mutex>

namespace ape {
namespace {
thread_local char g_err[512] = "";
}

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

namespace {

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// The kernels read and write rows with 16-byte vector accesses: every data pointer the host can
// see is checked (NULL passes: presence is checked where it matters).
inline bool misaligned(const void* p) { return ((uintptr_t)p & 15) != 0; }
#define APE_CHECK_ALIGNED(...)                                                                              \
    do {                                                                                                    \
        const void* ptrs_[] = {__VA_ARGS__};                                                                \
        for (const void* p_ : ptrs_)                                                                        \
            if (misaligned(p_)) return fail(APE_ERR_INVALID_ARG, "data pointer %p is not 16-byte aligned (%s)", p_, #__VA_ARGS__); \
    } while (0)
inline int ceil_div(long a, long b) { return (int)((a + b - 1) / b); }

}  // namespace

int check_shape(const ape_shape* s, ShapeInfo* o) {
    if (!s) return fail(APE_ERR_INVALID_ARG, "shape is NULL");
    o->hq = s->n_q_heads; o->hkv = s->n_kv_heads; o->d = s->head_dim;
    o->force_generic = (s->dtype & APE_DTYPE_FLAG_GENERIC) != 0;
    o->dtype = s->dtype & ~APE_DTYPE_FLAG_GENERIC;
    if (o->hq <= 0 || o->hkv <= 0 || o->d <= 0)
        return fail(APE_ERR_INVALID_ARG, "head counts and head_dim must be positive (got %d, %d, %d)", o->hq, o->hkv, o->d);
    if (o->hq % o->hkv) return fail(APE_ERR_INVALID_ARG, "n_q_heads %d is not a multiple of n_kv_heads %d", o->hq, o->hkv);
    if (o->dtype != APE_F32 && o->dtype != APE_BF16) return fail(APE_ERR_UNSUPPORTED, "dtype %d is not APE_F32 or APE_BF16", o->dtype);
    if (o->d > 256 || o->d % 8) return fail(APE_ERR_UNSUPPORTED, "head_dim %d: must be a multiple of 8 and <= 256", o->d);
    o->group = o->hq / o->hkv;
    o->mfma = !o->force_generic && o->dtype == APE_BF16 && o->d == 128 &&
              (o->group == 1 || o->group == 2 || o->group == 4 || o->group == 8);
    return APE_OK;
}

namespace {

int check_request(const ape_request* r, int q_len, int idx) {
    if (r->prefix_len < 0) return fail(APE_ERR_INVALID_ARG, "request %d: prefix_len %d < 0", idx, r->prefix_len);
    if (r->prefix_len > 0 && (!r->k_prefix || !r->v_prefix)) return fail(APE_ERR_INVALID_ARG, "request %d: prefix KV is NULL", idx);
    if (r->n_chunks < 0 || r->total_ctx_len < 0) return fail(APE_ERR_INVALID_ARG, "request %d: negative chunk count or context length", idx);
    if (r->n_chunks == 0 && r->total_ctx_len != 0) return fail(APE_ERR_INVALID_ARG, "request %d: total_ctx_len %d with no chunks", idx, r->total_ctx_len);
    if (r->n_chunks > 0 && (!r->k_chunks || !r->v_chunks || !r->cu_chunk_lens))
        return fail(APE_ERR_INVALID_ARG, "request %d: chunk table is NULL", idx);
    if (r->self_len < q_len || q_len < 1) return fail(APE_ERR_INVALID_ARG, "request %d: self_len %d < q_len %d (the query rows' own KV belongs to k_self)", idx, r->self_len, q_len);
    if (!r->k_self || !r->v_self) return fail(APE_ERR_INVALID_ARG, "request %d: self KV is NULL", idx);
    APE_CHECK_ALIGNED(r->k_prefix, r->v_prefix, r->k_self, r->v_self);
    if (((uintptr_t)r->k_chunks | (uintptr_t)r->v_chunks) & 7 || (uintptr_t)r->cu_chunk_lens & 3)
        return fail(APE_ERR_INVALID_ARG, "request %d: the chunk tables are not aligned to their element size", idx);
    if (!(std::isfinite(r->temperature) && r->temperature > 0.f)) return fail(APE_ERR_INVALID_ARG, "request %d: temperature must be finite and > 0", idx);
    if (!(std::isfinite(r->scale) && r->scale > 0.f)) return fail(APE_ERR_INVALID_ARG, "request %d: scale must be finite and > 0", idx);
    return APE_OK;
}

// Launch sizes: a grid times its workgroup size must stay below 2^32 work items and every count the
// kernels index with fits an int.  Calls beyond that are refused here, before any size is narrowed.
constexpr long kMaxUnits = 1L << 24;            // a query call writes FEWER (row, head) outputs than this: one 256-thread workgroup each in the merge
constexpr long kMaxTreeBlocks = 1L << 24;       // workgroups of the attention launch of a tree call (256 threads each)
constexpr long kMaxEncodeBlocks = 1L << 24;     // workgroups of the matrix-core encode (256 threads each)
constexpr long kMaxEncodeUnits = 1L << 26;      // (row, head) outputs of the generic encode: one wavefront each
}  // namespace

int check_encode_size(const ShapeInfo& si, int n_chunks, int max_len, long total_rows) {
    if (si.mfma) {
        // as launch_flash_encode sizes its grid, for the narrower of its two query tiles
        const long n_qtiles = ((long)max_len * si.group + 127) / 128;
        const long blocks = ((long)n_chunks * si.hkv + 7) / 8 * 8 * n_qtiles;
        if (blocks >= kMaxEncodeBlocks)
            return fail(APE_ERR_UNSUPPORTED, "encode of %d contexts of up to %d tokens needs %ld workgroups, fewer than %ld are supported "
                        "(the grid is contexts x KV heads x query tiles of the longest context: split the call)", n_chunks, max_len, blocks, kMaxEncodeBlocks);
    } else if (total_rows * si.hq >= kMaxEncodeUnits) {
        return fail(APE_ERR_UNSUPPORTED, "encode of %ld rows x %d heads on the generic path, fewer than %ld outputs are supported", total_rows, si.hq, kMaxEncodeUnits);
    }
    return APE_OK;
}

namespace {

KvView to_view(const ape_request* r) {
    KvView v;
    v.k_prefix = r->k_prefix; v.v_prefix = r->v_prefix;
    v.k_chunks = r->k_chunks; v.v_chunks = r->v_chunks; v.cu = r->cu_chunk_lens;
    v.k_self = r->k_self; v.v_self = r->v_self;
    v.prefix_len = r->prefix_len; v.n_chunks = r->n_chunks;
    v.total_ctx = r->n_chunks > 0 ? r->total_ctx_len : 0;
    v.self_len = r->self_len;
    v.temperature = r->temperature; v.scale = r->scale;
    return v;
}

// Number of context splits: enough workgroups to fill 256 CUs a few times over, never more than
// kMaxSplits, never splits shorter than `min_len` tokens.  Depends on sizes only.
QueryPlan plan_query(int base_workgroups, long max_ctx, int min_len, int target_workgroups) {
    QueryPlan p{};
    if (max_ctx <= 0) { p.n_ctx_splits = 0; p.ctx_split_len = 64; p.n_splits_total = 1; return p; }
    int want = ceil_div(target_workgroups, base_workgroups > 0 ? base_workgroups : 1);
    int cap = ceil_div(max_ctx, min_len);
    int n = want < 1 ? 1 : want;
    if (n > cap) n = cap;
    if (n > kMaxSplits) n = kMaxSplits;
    p.n_bound = n;                                     // rounding the length up to whole tiles can only lower the count
    long len = (max_ctx + n - 1) / n;
    len = (len + 63) / 64 * 64;                        // tiles never straddle a split
    n = ceil_div(max_ctx, len);
    p.n_ctx_splits = n; p.ctx_split_len = (int)len; p.n_splits_total = n + 1;
    return p;
}

// Split plan of a decode step.  Matrix-core path: one workgroup per (request, KV head, split), two
// of them resident per CU.  What decides the rate is how evenly the long (context) workgroups fill the
// 256 CUs: a count that is a multiple of 256 streams at 81-84 % of the HBM peak (256 itself is best:
// one long workgroup per CU, the short prefix+self ones run beside them), other counts at 72-79 %
// (32 requests x 16K: 1 / 2 / 3 / 4 / 8 splits = 84.1 / 82.2 / 76.0 / 80.4 / 80.2 %; 48 requests: 1 / 2 / 4 =
// 72.1 / 82.0 / 78.9 %; 16 requests: 1 / 2 / 4 = 57.2 / 83.1 / 78.4 %).  So: the smallest number of splits
// that makes requests x KV heads x splits a multiple of 256, if the splits stay at 256 tokens or more
// and the count at 2048 or less; otherwise many workgroups (at least 8 splits per request, about
// 2048 workgroups), where the remainder of the last round matters less.
QueryPlan decode_plan(const ShapeInfo& si, int batch, long max_ctx) {
    if (!si.mfma) return plan_query(batch * si.hq, max_ctx, 256, 1024);
    const int base = batch * si.hkv;
    int g = base, r = 256;
    while (r != 0) { const int t = g % r; g = r; r = t; }          // g = gcd(base, 256)
    const int n_even = 256 / g;
    if ((long)n_even * 256 <= (max_ctx > 256 ? max_ctx : 256) && n_even <= kMaxSplits && (long)base * n_even <= 2048)
        return plan_query(base, max_ctx, 256, base * n_even);
    const int want = ceil_div(2048, base);
    return plan_query(base, max_ctx, 256, (want < 8 ? 8 : want) * base);
}

// Split plan of the query prefill.  Matrix-core path: about one workgroup per CU (two of the narrow
// tile for contexts of middle length), the query tile chosen by flash_prefill_block_rows.
QueryPlan prefill_plan(const ShapeInfo& si, int batch, int q_len, long max_ctx) {
    const int rows = q_len * si.group;
    const long units = (long)batch * q_len * si.hq;
    const int bm = si.mfma ? flash_prefill_block_rows(rows, max_ctx) : 0;
    const int base = si.mfma ? batch * si.hkv * ceil_div(rows, bm) : (int)units;
    int target = si.mfma ? flash_prefill_target_workgroups(rows, max_ctx) : 1024;
    // Two workgroups per CU only pay when their streams stay long: with few query rows (few row tiles)
    // the same target cuts the context into splits of a few hundred tokens, whose fixed cost per
    // workgroup outweighs the second workgroup (64 rows over 16K: 0.049 ms with 32 splits of 512 tokens,
    // 0.036 ms with 16 of 1024).
    if (si.mfma && target > 256 && max_ctx / ceil_div(target, base) < 2048) target = 256;
    QueryPlan p = plan_query(base, max_ctx, 256, target);
    p.block_rows = bm;
    return p;
}

// Splits of the tree entry point: the contexts of every node that holds contexts are cut into
// runs of `len` tokens; `len` is what the flat entry points would use for the same sizes, so a
// one-node tree runs exactly like them.  max_splits bounds the splits in use from sizes only:
// sum over such nodes of ceil(tokens / len) <= total / len + number of nodes.
struct TreePlan {
    int len;
    int max_splits;
    int block_rows;        // query tile of the flash prefill (see QueryPlan)
    size_t partial_bytes, plan_bytes;
};

TreePlan plan_tree(const ShapeInfo& si, long total_ctx, int n_nodes, int q_len) {
    QueryPlan qp;
    if (q_len == 1) qp = decode_plan(si, 1, total_ctx);
    else qp = prefill_plan(si, 1, q_len, total_ctx);
    TreePlan p;
    p.len = qp.ctx_split_len;
    p.block_rows = qp.block_rows;
    p.max_splits = ceil_div(total_ctx > 0 ? total_ctx : 1, p.len) + n_nodes;
    const long units = (long)q_len * si.hq;
    p.partial_bytes = align_up((size_t)units * (p.max_splits + 1) * si.d * sizeof(float), kWsAlign) +
                      align_up((size_t)units * (p.max_splits + 1) * sizeof(float), kWsAlign);
    p.plan_bytes = align_up((size_t)TreePlanLayout{n_nodes, p.max_splits}.words() * sizeof(int32_t), kWsAlign);
    return p;
}

// Checks the numbering rules of ape_tree_node and finds the level ranges.
int check_tree(const ape_tree_node* nodes, int n_nodes, int n_chunks, int* n_levels, int32_t* level_start) {
    if (!nodes) return fail(APE_ERR_INVALID_ARG, "tree nodes are NULL");
    if (n_nodes < 1) return fail(APE_ERR_INVALID_ARG, "a tree needs at least one node (got %d)", n_nodes);
    if (n_nodes > APE_TREE_MAX_NODES) return fail(APE_ERR_UNSUPPORTED, "%d tree nodes, at most %d are supported", n_nodes, APE_TREE_MAX_NODES);
    if (n_chunks < 1) return fail(APE_ERR_INVALID_ARG, "a tree needs at least one context");
    if (n_chunks > APE_TREE_MAX_CONTEXTS) return fail(APE_ERR_UNSUPPORTED, "%d contexts, at most %d are supported under a tree", n_chunks, APE_TREE_MAX_CONTEXTS);
    bool owned[APE_TREE_MAX_CONTEXTS] = {};            // on the stack: the call allocates nothing, on the host either
    long next_child = 1;
    for (int n = 0; n < n_nodes; ++n) {
        const ape_tree_node& t = nodes[n];
        if (!(std::isfinite(t.scale) && t.scale > 0.f)) return fail(APE_ERR_INVALID_ARG, "tree node %d: scale must be finite and > 0", n);
        if (t.count < 1) return fail(APE_ERR_INVALID_ARG, "tree node %d: count %d < 1", n, t.count);
        if (t.leaf_children) {
            if (t.first < 0 || (long)t.first + t.count > n_chunks) return fail(APE_ERR_INVALID_ARG, "tree node %d: contexts %d..%ld are outside the chunk table of %d", n, t.first, (long)t.first + t.count - 1, n_chunks);
            for (int i = 0; i < t.count; ++i) {
                if (owned[t.first + i]) return fail(APE_ERR_INVALID_ARG, "tree node %d: context %d already belongs to another node", n, t.first + i);
                owned[t.first + i] = 1;
            }
        } else {
            if (t.first != next_child) return fail(APE_ERR_INVALID_ARG, "tree node %d: node children must start at %ld (breadth-first numbering), got %d", n, next_child, t.first);
            next_child += t.count;
            if (next_child > n_nodes) return fail(APE_ERR_INVALID_ARG, "tree node %d: children run past the %d nodes given", n, n_nodes);
        }
    }
    if (next_child != n_nodes) return fail(APE_ERR_INVALID_ARG, "%ld of the %d nodes are reachable from the root", next_child, n_nodes);
    for (int c = 0; c < n_chunks; ++c)
        if (!owned[c]) return fail(APE_ERR_INVALID_ARG, "context %d belongs to no tree node", c);
    // levels: the node children of one level are the next level, and they are contiguous
    int lv = 0;
    level_start[0] = 0; level_start[1] = 1;
    while (true) {
        long kids = 0;
        for (int n = level_start[lv]; n < level_start[lv + 1]; ++n)
            if (!nodes[n].leaf_children) kids += nodes[n].count;
        if (kids == 0) break;
        if (lv + 1 >= kMaxTreeLevels) return fail(APE_ERR_UNSUPPORTED, "the tree is deeper than %d levels of nodes", kMaxTreeLevels);
        ++lv;
        level_start[lv + 1] = level_start[lv] + (int32_t)kids;
    }
    *n_levels = lv + 1;
    return APE_OK;
}

size_t partial_bytes(long units, int n_splits_total, int d) {
    return align_up((size_t)units * n_splits_total * d * sizeof(float), kWsAlign) +
           align_up((size_t)units * n_splits_total * sizeof(float), kWsAlign);
}

}  // namespace
}  // namespace ape

using namespace ape;

extern "C" {

const char* ape_status_string(int status) {
    switch (status) {
        case APE_OK: return "ok";
        case APE_ERR_INVALID_ARG: return "invalid argument";
        case APE_ERR_UNSUPPORTED: return "unsupported shape or dtype";
        case APE_ERR_WORKSPACE: return "workspace missing or too small";
        case APE_ERR_DEVICE: return "HIP launch error";
        default: return "unknown status";
    }
}

const char* ape_last_error(void) { return g_err; }
const char* ape_version(void) { return "0.1.0"; }

size_t ape_workspace_bytes(int op, const ape_shape* shape, int32_t batch, int32_t q_len, int64_t max_total_kv) {
    ShapeInfo si;
    if (check_shape(shape, &si) != APE_OK) return 0;
    if (op == APE_OP_ENCODE) return 0;
    if (op == APE_OP_DECODE) q_len = 1;
    else if (op != APE_OP_PREFILL) return 0;
    if (batch < 1 || q_len < 1) return 0;
    if ((long)batch * q_len * si.hq >= kMaxUnits) return 0;     // the entry points refuse such a call
    // The most context splits any call can ask for whose longest context has at most max_total_kv
    // tokens (negative: any length), + 1 for prefix + self.  Decode: the count only grows with the
    // length.  Prefill: the plan changes its query tile and its workgroup target with the context
    // length; within each of the three ranges the count before rounding only grows with the length,
    // so the upper ends of the ranges below the cap, and the cap itself, decide.
    const long any_len = (long)kMaxSplits * (1 << 20);
    const long cap = max_total_kv < 0 || max_total_kv > any_len ? any_len : (long)max_total_kv;
    int n_max = 0;
    if (op == APE_OP_DECODE) {
        n_max = decode_plan(si, batch, cap).n_bound;
    } else {
        for (long ctx : {kPrefillOneWorkgroupPerCuMaxCtx, flash_prefill_narrow_tile_max_ctx(q_len * si.group), cap}) {
            if (ctx > cap) continue;
            const int n = prefill_plan(si, batch, q_len, ctx).n_bound;
            if (n > n_max) n_max = n;
        }
    }
    return partial_bytes((long)batch * q_len * si.hq, n_max + 1, si.d);
}

int ape_encode_chunks(const ape_shape* shape,
                      const void* q_prefix, const void* k_prefix, const void* v_prefix, int32_t prefix_len,
                      const void* q_chunks, const void* k_chunks, const void* v_chunks,
                      const int32_t* cu_host, const int32_t* cu_dev, int32_t n_chunks,
                      void* o_prefix, void* o_chunks, float* lse_prefix, float* lse_chunks,
                      void* workspace, size_t workspace_bytes, void* stream) {
    (void)workspace; (void)workspace_bytes;
    ShapeInfo si;
    int rc = check_shape(shape, &si);
    if (rc) return rc;
    if (prefix_len < 0 || n_chunks < 0) return fail(APE_ERR_INVALID_ARG, "prefix_len and n_chunks must be >= 0");
    if (prefix_len > 0 && (!k_prefix || !v_prefix)) return fail(APE_ERR_INVALID_ARG, "prefix KV is NULL");
    if ((q_prefix == nullptr) != (o_prefix == nullptr)) return fail(APE_ERR_INVALID_ARG, "q_prefix and o_prefix must both be given or both be NULL");
    if (lse_prefix && !q_prefix) return fail(APE_ERR_INVALID_ARG, "lse_prefix given without q_prefix");
    APE_CHECK_ALIGNED(q_prefix, k_prefix, v_prefix, q_chunks, k_chunks, v_chunks, o_prefix, o_chunks);
    long total = 0;
    int max_len = 0, min_len = INT32_MAX;
    if (n_chunks > 0) {
        if (!cu_host || !cu_dev) return fail(APE_ERR_INVALID_ARG, "cu_chunk_lens (host and device) are required");
        if (cu_host[0] != 0) return fail(APE_ERR_INVALID_ARG, "cu_chunk_lens[0] must be 0");
        for (int i = 0; i < n_chunks; ++i) {
            const long li = (long)cu_host[i + 1] - cu_host[i];
            if (li < 0) return fail(APE_ERR_INVALID_ARG, "cu_chunk_lens is not non-decreasing at %d", i);
            if (li > max_len) max_len = (int)li;
            if (li < min_len) min_len = (int)li;
        }
        total = cu_host[n_chunks];
        if (total > 0 && (!q_chunks || !k_chunks || !v_chunks || !o_chunks)) return fail(APE_ERR_INVALID_ARG, "chunk Q/K/V/O is NULL");
        rc = check_encode_size(si, n_chunks, max_len, total);
        if (rc) return rc;
    }
    if (q_prefix && prefix_len > 0) {
        rc = check_encode_size(si, 1, prefix_len, prefix_len);
        if (rc) return rc;
    }
    hipStream_t st = (hipStream_t)stream;

    // the prefix rows are one more "context" with no prefix in front of it
    if (q_prefix && prefix_len > 0) {
        // cu for a single chunk [0, prefix_len): reuse of a device table is not possible without a
        // copy, so the prefix rows go through the kernels' single-chunk mode (cu == NULL).
        EncodeArgs e{};
        e.q = q_prefix; e.k = k_prefix; e.v = v_prefix; e.k_prefix = nullptr; e.v_prefix = nullptr;
        e.cu = nullptr; e.out = o_prefix; e.lse = lse_prefix;
        e.n_chunks = 1; e.prefix_len = 0; e.total_rows = prefix_len; e.max_chunk_len = prefix_len;
        e.n_q_heads = si.hq; e.n_kv_heads = si.hkv; e.head_dim = si.d;
        hipError_t he = si.mfma ? launch_flash_encode(e, st) : launch_generic_encode(e, si.dtype, st);
        if (he != hipSuccess) return fail(APE_ERR_DEVICE, "encode (prefix rows): %s", hipGetErrorString(he));
    }
    if (total > 0) {
        EncodeArgs e{};
        e.q = q_chunks; e.k = k_chunks; e.v = v_chunks; e.k_prefix = k_prefix; e.v_prefix = v_prefix;
        e.cu = cu_dev; e.out = o_chunks; e.lse = lse_chunks;
        e.n_chunks = n_chunks; e.prefix_len = prefix_len; e.total_rows = (int)total; e.max_chunk_len = max_len;
        e.n_q_heads = si.hq; e.n_kv_heads = si.hkv; e.head_dim = si.d;
        e.uniform_chunks = min_len == max_len;
        hipError_t he = si.mfma ? launch_flash_encode(e, st) : launch_generic_encode(e, si.dtype, st);
        if (he != hipSuccess) return fail(APE_ERR_DEVICE, "encode: %s", hipGetErrorString(he));
    }
    return APE_OK;
}

// `static_limit`: the workspace is the library's own fixed array, so a call that needs more is one
// the entry point does not support (rather than a caller's buffer being too small).
static int run_query(const ShapeInfo& si, const ape_request* reqs, int batch, int q_len, bool decode,
                     const void* q, void* out, float* lse_out, void* workspace, size_t workspace_bytes, hipStream_t st,
                     bool static_limit = false) {
    long max_ctx = 0;
    for (int b = 0; b < batch; ++b) {
        int rc = check_request(&reqs[b], q_len, b);
        if (rc) return rc;
        const long m = reqs[b].n_chunks > 0 ? reqs[b].total_ctx_len : 0;
        if (m > max_ctx) max_ctx = m;
    }
    APE_CHECK_ALIGNED(q, out);
    const long units = (long)batch * q_len * si.hq;
    if (units >= kMaxUnits)
        return fail(APE_ERR_UNSUPPORTED, "%d requests x %d rows x %d heads = %ld outputs in one call, fewer than %ld are supported", batch, q_len, si.hq, units, kMaxUnits);
    QueryPlan plan;
    if (decode) {
        plan = decode_plan(si, batch, max_ctx);
    } else {
        plan = prefill_plan(si, batch, q_len, max_ctx);
    }
    const size_t need = partial_bytes(units, plan.n_splits_total, si.d);
    if (static_limit && workspace_bytes < need)
        return fail(APE_ERR_UNSUPPORTED, "%d requests x %d heads over up to %ld context tokens need %zu bytes of partial results; the "
                    "built-in buffer holds %zu (use ape_attention_decode with a workspace of the caller's)", batch, si.hq, max_ctx, need, workspace_bytes);
    if (!workspace || workspace_bytes < need)
        return fail(APE_ERR_WORKSPACE, "workspace of %zu bytes given, %zu needed (ape_workspace_bytes gives the bound)", workspace_bytes, need);
    if ((uintptr_t)workspace % kWsAlign) return fail(APE_ERR_WORKSPACE, "workspace must be %d-byte aligned", kWsAlign);
    float* part_o = (float*)workspace;
    float* part_lse = (float*)((char*)workspace + align_up((size_t)units * plan.n_splits_total * si.d * sizeof(float), kWsAlign));

    for (int b0 = 0; b0 < batch; b0 += kMaxReqPerLaunch) {
        const int nb = batch - b0 < kMaxReqPerLaunch ? batch - b0 : kMaxReqPerLaunch;
        QueryArgs a{};
        MergeArgs m{};
        for (int i = 0; i < nb; ++i) {
            a.req[i] = to_view(&reqs[b0 + i]);
            m.scale[i] = reqs[b0 + i].scale;
            m.total_ctx[i] = a.req[i].total_ctx;
        }
        m.ctx_split_len = plan.ctx_split_len;
        a.q = (const char*)q + (size_t)b0 * q_len * si.hq * si.d * (si.dtype == APE_F32 ? 4 : 2);
        a.part_o = part_o; a.part_lse = part_lse;
        a.n_req = nb; a.q_len = q_len; a.n_q_heads = si.hq; a.n_kv_heads = si.hkv; a.head_dim = si.d;
        a.n_ctx_splits = plan.n_ctx_splits; a.ctx_split_len = plan.ctx_split_len;
        a.units_total = (int)units; a.req_base = b0;
        hipError_t he;
        // (a decode step is a query of one row: the flash kernel's narrow tile, one wavefront computing)
        if (si.mfma) he = launch_flash_prefill(a, decode ? 128 : plan.block_rows, st);
        else he = launch_generic_query(a, si.dtype, st);
        if (he != hipSuccess) return fail(APE_ERR_DEVICE, "attention kernel: %s", hipGetErrorString(he));

        m.part_o = part_o; m.part_lse = part_lse; m.out = out; m.lse_out = lse_out;
        m.n_req = nb; m.q_len = q_len; m.n_q_heads = si.hq; m.head_dim = si.d;
        m.n_ctx_splits = plan.n_ctx_splits; m.n_splits_total = plan.n_splits_total;
        m.units_total = (int)units; m.req_base = b0; m.lse_head_major = decode ? 0 : 1; m.dtype = si.dtype;
        he = launch_merge(m, st);
        if (he != hipSuccess) return fail(APE_ERR_DEVICE, "merge kernel: %s", hipGetErrorString(he));
    }
    return APE_OK;
}

int ape_attention_prefill(const ape_shape* shape, const ape_request* req,
                          const void* q, int32_t q_len, void* out, float* lse_out,
                          void* workspace, size_t workspace_bytes, void* stream) {
    ShapeInfo si;
    int rc = check_shape(shape, &si);
    if (rc) return rc;
    if (!req || !q || !out) return fail(APE_ERR_INVALID_ARG, "req, q and out must not be NULL");
    if (q_len < 1) return fail(APE_ERR_INVALID_ARG, "q_len %d < 1", q_len);
    return run_query(si, req, 1, q_len, false, q, out, lse_out, workspace, workspace_bytes, (hipStream_t)stream);
}

int ape_attention_prefill_batch(const ape_shape* shape, const ape_request* reqs, int32_t batch,
                                const void* q, int32_t q_len, void* out, float* lse_out,
                                void* workspace, size_t workspace_bytes, void* stream) {
    ShapeInfo si;
    int rc = check_shape(shape, &si);
    if (rc) return rc;
    if (!reqs || !q || !out) return fail(APE_ERR_INVALID_ARG, "reqs, q and out must not be NULL");
    if (batch < 1) return fail(APE_ERR_INVALID_ARG, "batch %d < 1", batch);
    if (q_len < 1) return fail(APE_ERR_INVALID_ARG, "q_len %d < 1", q_len);
    return run_query(si, reqs, batch, q_len, false, q, out, lse_out, workspace, workspace_bytes, (hipStream_t)stream);
}

int ape_attention_decode(const ape_shape* shape, const ape_request* reqs, int32_t batch,
                         const void* q, void* out, float* lse_out,
                         void* workspace, size_t workspace_bytes, void* stream) {
    ShapeInfo si;
    int rc = check_shape(shape, &si);
    if (rc) return rc;
    if (!reqs || !q || !out) return fail(APE_ERR_INVALID_ARG, "reqs, q and out must not be NULL");
    if (batch < 1) return fail(APE_ERR_INVALID_ARG, "batch %d < 1", batch);
    return run_query(si, reqs, batch, 1, true, q, out, lse_out, workspace, workspace_bytes, (hipStream_t)stream);
}

// ---- decode with the partial results in a buffer of the library's own -----------------------
// The array lives in every GPU's memory from the moment the library is loaded there until the
// process ends.  In host code its name is only a handle: the address a kernel can use comes from
// hipGetSymbolAddress, once per device (each GPU has its own copy at its own address).
static __device__ __align__(256) unsigned char scratch[APE_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (resolved at the first call there).
int static_scratch(void** out) {
    int dev = -1;
    hipError_t he = hipGetDevice(&dev);
    if (he != hipSuccess) return fail(APE_ERR_DEVICE, "hipGetDevice: %s", hipGetErrorString(he));
    if (dev < 0 || dev >= kMaxDevices) return fail(APE_ERR_UNSUPPORTED, "device index %d, at most %d devices are supported", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        he = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (he != hipSuccess || !p) return fail(APE_ERR_DEVICE, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(he));
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return APE_OK;
}
}  // namespace

int ape_attention_decode_static(const ape_shape* shape, const ape_request* reqs, int32_t batch,
                                const void* q, void* out, float* lse_out, void* stream) {
    ShapeInfo si;
    int rc = check_shape(shape, &si);
    if (rc) return rc;
    if (!reqs || !q || !out) return fail(APE_ERR_INVALID_ARG, "reqs, q and out must not be NULL");
    if (batch < 1) return fail(APE_ERR_INVALID_ARG, "batch %d < 1", batch);
    void* ws = nullptr;
    rc = static_scratch(&ws);
    if (rc) return rc;
    // Nothing in the buffer has to start at zero: every partial result the merge reads is written
    // by the attention kernel of the same call (the merge stops at each request's last split).
    return run_query(si, reqs, batch, 1, true, q, out, lse_out, ws, (size_t)APE_STATIC_SCRATCH_BYTES, (hipStream_t)stream, true);
}

size_t ape_tree_workspace_bytes(const ape_shape* shape, int32_t total_ctx_len, int32_t n_nodes, int32_t q_len) {
    ShapeInfo si;
    if (check_shape(shape, &si) != APE_OK) return 0;
    if (total_ctx_len < 0 || n_nodes < 1 || n_nodes > APE_TREE_MAX_NODES || q_len < 1) return 0;
    const TreePlan p = plan_tree(si, total_ctx_len, n_nodes, q_len);
    if (p.max_splits > kMaxTreeSplits) return 0;
    return p.partial_bytes + p.plan_bytes;
}

int ape_attention_tree(const ape_shape* shape, const ape_request* req,
                       const ape_tree_node* nodes_host, const ape_tree_node* nodes_dev, int32_t n_nodes,
                       const void* q, int32_t q_len, void* out, float* lse_out,
                       void* workspace, size_t workspace_bytes, void* stream) {
    ShapeInfo si;
    int rc = check_shape(shape, &si);
    if (rc) return rc;
    if (!req || !q || !out) return fail(APE_ERR_INVALID_ARG, "req, q and out must not be NULL");
    if (q_len < 1) return fail(APE_ERR_INVALID_ARG, "q_len %d < 1", q_len);
    rc = check_request(req, q_len, 0);
    if (rc) return rc;
    APE_CHECK_ALIGNED(q, out);
    if ((long)q_len * si.hq >= kMaxUnits)
        return fail(APE_ERR_UNSUPPORTED, "%d rows x %d heads = %ld outputs in one call, fewer than %ld are supported", q_len, si.hq, (long)q_len * si.hq, kMaxUnits);
    TreeMergeArgs m{};
    rc = check_tree(nodes_host, n_nodes, req->n_chunks, &m.n_levels, m.level_start);
    if (rc) return rc;
    if (!nodes_dev) return fail(APE_ERR_INVALID_ARG, "the device copy of the tree nodes is NULL");

    const TreePlan plan = plan_tree(si, req->total_ctx_len, n_nodes, q_len);
    if (plan.max_splits > kMaxTreeSplits)
        return fail(APE_ERR_UNSUPPORTED, "%d splits would be needed, at most %d are supported", plan.max_splits, kMaxTreeSplits);
    const long units = (long)q_len * si.hq;
    // The attention grid is sized from the bound on the splits, not from the splits in use: one
    // workgroup of 256 threads per (split slot, KV head[, query tile]); its work items must stay
    // below 2^32.
    {
        const long slots = (long)plan.max_splits + 1;
        long blocks;
        if (si.mfma && q_len > 1) {
            const long n_qtiles = ((long)q_len * si.group + plan.block_rows - 1) / plan.block_rows;
            blocks = ((slots - 1) * si.hkv + 7) / 8 * 8 * n_qtiles + ((long)si.hkv + 7) / 8 * 8 * n_qtiles;
        } else if (si.mfma) {
            blocks = slots * si.hkv;
        } else {
            blocks = slots * units;
        }
        if (blocks >= kMaxTreeBlocks)
            return fail(APE_ERR_UNSUPPORTED, "the tree call would launch %ld workgroups (%d split slots x heads x query tiles), fewer than %ld are "
                        "supported: fewer nodes or fewer query rows per call", blocks, plan.max_splits + 1, kMaxTreeBlocks);
    }
    const size_t need = plan.partial_bytes + plan.plan_bytes;
    if (!workspace || workspace_bytes < need)
        return fail(APE_ERR_WORKSPACE, "workspace of %zu bytes given, %zu needed (ape_tree_workspace_bytes gives the size)", workspace_bytes, need);
    if ((uintptr_t)workspace % kWsAlign) return fail(APE_ERR_WORKSPACE, "workspace must be %d-byte aligned", kWsAlign);
    float* part_o = (float*)workspace;
    float* part_lse = (float*)((char*)workspace + align_up((size_t)units * (plan.max_splits + 1) * si.d * sizeof(float), kWsAlign));
    int32_t* plan_dev = (int32_t*)((char*)workspace + plan.partial_bytes);
    hipStream_t st = (hipStream_t)stream;

    TreePlanArgs tp{};
    tp.nodes = nodes_dev; tp.cu = req->cu_chunk_lens; tp.plan = plan_dev;
    tp.n_nodes = n_nodes; tp.max_splits = plan.max_splits; tp.split_len = plan.len;
    hipError_t he = launch_tree_plan(tp, st);
    if (he != hipSuccess) return fail(APE_ERR_DEVICE, "tree plan kernel: %s", hipGetErrorString(he));

    QueryArgs a{};
    a.req[0] = to_view(req);
    a.q = q; a.part_o = part_o; a.part_lse = part_lse;
    a.n_req = 1; a.q_len = q_len; a.n_q_heads = si.hq; a.n_kv_heads = si.hkv; a.head_dim = si.d;
    a.n_ctx_splits = plan.max_splits; a.ctx_split_len = plan.len;
    a.split_ranges = plan_dev + TreePlanLayout{n_nodes, plan.max_splits}.ranges_at();
    a.units_total = (int)units; a.req_base = 0;
    if (si.mfma) he = launch_flash_prefill(a, q_len == 1 ? 128 : plan.block_rows, st);
    else he = launch_generic_query(a, si.dtype, st);
    if (he != hipSuccess) return fail(APE_ERR_DEVICE, "attention kernel: %s", hipGetErrorString(he));

    m.part_o = part_o; m.part_lse = part_lse; m.out = out; m.lse_out = lse_out; m.nodes = nodes_dev; m.plan = plan_dev;
    m.n_nodes = n_nodes; m.max_splits = plan.max_splits; m.units_total = (int)units;
    m.q_len = q_len; m.n_q_heads = si.hq; m.head_dim = si.d; m.dtype = si.dtype;
    he = launch_tree_merge(m, st);
    if (he != hipSuccess) return fail(APE_ERR_DEVICE, "tree merge kernel: %s", hipGetErrorString(he));
    return APE_OK;
}

int ape_rope_write_cache(const ape_shape* shape,
                         const void* q_raw, const void* k_raw, const void* v_raw,
                         const int32_t* cu_host, const int32_t* cu_dev, int32_t n_chunks,
                         int32_t position_offset, float rope_base,
                         void* q_rot, void* const* k_cache, void* const* v_cache, void* stream) {
    ShapeInfo si;
    int rc = check_shape(shape, &si);
    if (rc) return rc;
    if (n_chunks < 0) return fail(APE_ERR_INVALID_ARG, "n_chunks %d < 0", n_chunks);
    if (position_offset < 0) return fail(APE_ERR_INVALID_ARG, "position_offset %d < 0", position_offset);
    if (!(std::isfinite(rope_base) && rope_base > 0.f)) return fail(APE_ERR_INVALID_ARG, "rope_base must be finite and > 0");
    if ((q_raw == nullptr) != (q_rot == nullptr)) return fail(APE_ERR_INVALID_ARG, "q_raw and q_rot must both be given or both be NULL");
    APE_CHECK_ALIGNED(q_raw, k_raw, v_raw, q_rot);
    if ((k_raw == nullptr) != (k_cache == nullptr)) return fail(APE_ERR_INVALID_ARG, "k_raw and k_cache must both be given or both be NULL");
    if ((v_raw == nullptr) != (v_cache == nullptr)) return fail(APE_ERR_INVALID_ARG, "v_raw and v_cache must both be given or both be NULL");
    if (n_chunks == 0) return APE_OK;
    if (!cu_host || !cu_dev) return fail(APE_ERR_INVALID_ARG, "cu_chunk_lens (host and device) are required");
    if (cu_host[0] != 0) return fail(APE_ERR_INVALID_ARG, "cu_chunk_lens[0] must be 0");
    for (int i = 0; i < n_chunks; ++i)
        if (cu_host[i + 1] < cu_host[i]) return fail(APE_ERR_INVALID_ARG, "cu_chunk_lens is not non-decreasing at %d", i);
    RopeArgs a{};
    a.q_raw = q_raw; a.k_raw = k_raw; a.v_raw = v_raw; a.q_rot = q_rot; a.k_cache = k_cache; a.v_cache = v_cache;
    a.cu = cu_dev; a.n_chunks = n_chunks; a.total_rows = cu_host[n_chunks];
    a.n_q_heads = si.hq; a.n_kv_heads = si.hkv; a.head_dim = si.d; a.position_offset = position_offset;
    a.q_stride = (int64_t)si.hq * si.d; a.k_stride = a.v_stride = (int64_t)si.hkv * si.d;
    for (int c = 0; c < si.d / 2; ++c) a.inv_freq[c] = std::pow((double)rope_base, -2.0 * c / si.d);
    hipError_t he = launch_rope_write(a, si.dtype, (hipStream_t)stream);
    if (he != hipSuccess) return fail(APE_ERR_DEVICE, "rope kernel: %s", hipGetErrorString(he));
    return APE_OK;
}

}  // extern "C"
