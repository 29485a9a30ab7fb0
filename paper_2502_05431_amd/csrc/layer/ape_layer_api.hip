// Host side of include/ape_layer.h: one transformer layer, and a stack of layers, around the
// block-diagonal encode attention of the context pre-caching pass (arXiv 2502.05431, Section 2.2;
// Section 5.4 measures this pass for whole models).  A separate shared object: it links rocBLAS
// and keeps a handle per device, which the attention library (libape_hip.so) must not.
#include "ape_layer_internal.h"

#include <cmath>

namespace ape {
namespace {

constexpr long kMlpSlabRows = 16384;           // rows of the MLP processed at a time (bounds the workspace)

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline bool misaligned(const void* p) { return ((uintptr_t)p & 15) != 0; }

struct LayerPlan {
    size_t h, qkv, q_rot, x1, gu, act, total;   // byte offsets into the workspace, and its size
    long slab;
};

LayerPlan plan_layer(const ShapeInfo& si, int hidden, int inter, long rows) {
    const size_t es = si.dtype == APE_F32 ? 4 : 2;
    LayerPlan p;
    p.slab = rows < kMlpSlabRows ? rows : kMlpSlabRows;
    size_t off = 0;
    auto take = [&](size_t elems) { const size_t at = off; off += align_up(elems * es, kWsAlign); return at; };
    p.h = take((size_t)rows * hidden);
    p.qkv = take((size_t)rows * (si.hq + 2 * si.hkv) * si.d);
    p.q_rot = take((size_t)rows * si.hq * si.d);
    p.x1 = take((size_t)rows * hidden);
    p.gu = take((size_t)p.slab * 2 * inter);
    p.act = take((size_t)p.slab * inter);
    p.total = off;
    return p;
}

int check_layer(const ape_layer_weights* w, int idx) {
    if (!w) return fail(APE_ERR_INVALID_ARG, "layer weights are NULL");
    if (w->hidden < 8 || w->hidden % 8 || w->intermediate < 8 || w->intermediate % 8)
        return fail(APE_ERR_UNSUPPORTED, "layer %d: hidden %d and intermediate %d must be positive multiples of 8", idx, w->hidden, w->intermediate);
    if (!(std::isfinite(w->rms_eps) && w->rms_eps >= 0.f)) return fail(APE_ERR_INVALID_ARG, "layer %d: rms_eps must be finite and >= 0", idx);
    if (!(std::isfinite(w->rope_base) && w->rope_base > 0.f)) return fail(APE_ERR_INVALID_ARG, "layer %d: rope_base must be finite and > 0", idx);
    if (!w->attn_norm || !w->w_qkv || !w->w_o || !w->mlp_norm || !w->w_gate_up || !w->w_down)
        return fail(APE_ERR_INVALID_ARG, "layer %d: a weight pointer is NULL", idx);
    for (const void* p : {w->attn_norm, w->w_qkv, w->w_o, w->mlp_norm, w->w_gate_up, w->w_down})
        if (misaligned(p)) return fail(APE_ERR_INVALID_ARG, "layer %d: weight pointer %p is not 16-byte aligned", idx, p);
    return APE_OK;
}

// What every layer of a call shares, checked once.
struct Contexts {
    const int32_t* cu_dev;
    int n_chunks, max_len, min_len, prefix_len;
    long rows;
};

int check_contexts(const ShapeInfo& si, int32_t prefix_len, const int32_t* cu_host, const int32_t* cu_dev, int32_t n_chunks, Contexts* c) {
    if (prefix_len < 0 || n_chunks < 0) return fail(APE_ERR_INVALID_ARG, "prefix_len and n_chunks must be >= 0");
    c->cu_dev = cu_dev; c->n_chunks = n_chunks; c->prefix_len = prefix_len; c->max_len = 0; c->min_len = INT32_MAX; c->rows = 0;
    if (n_chunks == 0) return APE_OK;
    if (!cu_host || !cu_dev) return fail(APE_ERR_INVALID_ARG, "cu_chunk_lens (host and device) are required");
    if (cu_host[0] != 0) return fail(APE_ERR_INVALID_ARG, "cu_chunk_lens[0] must be 0");
    for (int i = 0; i < n_chunks; ++i) {
        const long li = (long)cu_host[i + 1] - cu_host[i];
        if (li < 0) return fail(APE_ERR_INVALID_ARG, "cu_chunk_lens is not non-decreasing at %d", i);
        if (li > c->max_len) c->max_len = (int)li;
        if (li < c->min_len) c->min_len = (int)li;
    }
    c->rows = cu_host[n_chunks];
    return c->rows > 0 ? check_encode_size(si, n_chunks, c->max_len, c->rows) : APE_OK;
}

// One layer; everything has been validated.  The caller holds a BlasCall.
int run_layer(const ShapeInfo& si, const ape_layer_weights* w, const Contexts& c, const void* x,
              const void* k_prefix, const void* v_prefix, void* k_cache, void* v_cache, void* y,
              const ape_layer_taps* taps, char* ws, const LayerPlan& p, hipStream_t st) {
    const size_t es = si.dtype == APE_F32 ? 4 : 2;
    const long rows = c.rows;
    void *h = ws + p.h, *qkv = ws + p.qkv, *x1 = ws + p.x1, *gu = ws + p.gu, *act = ws + p.act;
    void* q_rot = taps && taps->q_rot ? taps->q_rot : (void*)(ws + p.q_rot);
    const int hidden = w->hidden, inter = w->intermediate;
    const int qd = si.hq * si.d, kvd = si.hkv * si.d, qkvd = qd + 2 * kvd;
    auto dev_fail = [&](const char* what, hipError_t e) { return fail(APE_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e)); };

    // attention half: norm -> QKV -> rotary embedding + cache write -> attention -> output projection + residual
    hipError_t he = launch_rmsnorm(x, w->attn_norm, h, rows, hidden, w->rms_eps, si.dtype, st);
    if (he != hipSuccess) return dev_fail("RMSNorm", he);
    if (gemm_xwT(h, hidden, w->w_qkv, nullptr, qkv, qkvd, rows, qkvd, hidden, si.dtype, st)) return fail(APE_ERR_DEVICE, "QKV projection (rocBLAS) failed");
    RopeArgs ra{};
    ra.q_raw = qkv; ra.k_raw = (char*)qkv + (size_t)qd * es; ra.v_raw = (char*)qkv + (size_t)(qd + kvd) * es;
    ra.q_rot = q_rot; ra.k_packed = k_cache; ra.v_packed = v_cache;
    ra.q_stride = ra.k_stride = ra.v_stride = qkvd;
    ra.cu = c.cu_dev; ra.n_chunks = c.n_chunks; ra.total_rows = (int)rows;
    ra.n_q_heads = si.hq; ra.n_kv_heads = si.hkv; ra.head_dim = si.d; ra.position_offset = c.prefix_len;
    for (int ch = 0; ch < si.d / 2; ++ch) ra.inv_freq[ch] = std::pow((double)w->rope_base, -2.0 * ch / si.d);
    he = launch_rope_write(ra, si.dtype, st);
    if (he != hipSuccess) return dev_fail("rotary embedding", he);
    void* attn = taps && taps->attn ? taps->attn : qkv;  // (the raw projections are no longer needed)
    EncodeArgs e{};
    e.q = q_rot; e.k = k_cache; e.v = v_cache; e.k_prefix = k_prefix; e.v_prefix = v_prefix;
    e.cu = c.cu_dev; e.out = attn; e.lse = nullptr;
    e.n_chunks = c.n_chunks; e.prefix_len = c.prefix_len; e.total_rows = (int)rows; e.max_chunk_len = c.max_len;
    e.n_q_heads = si.hq; e.n_kv_heads = si.hkv; e.head_dim = si.d; e.uniform_chunks = c.min_len == c.max_len;
    he = si.mfma ? launch_flash_encode(e, st) : launch_generic_encode(e, si.dtype, st);
    if (he != hipSuccess) return dev_fail("encode attention", he);
    if (gemm_xwT(attn, qd, w->w_o, x, x1, hidden, rows, hidden, qd, si.dtype, st)) return fail(APE_ERR_DEVICE, "output projection (rocBLAS) failed");

    // MLP half, a slab of rows at a time: norm -> gate/up -> SiLU(gate) * up -> down projection + residual
    he = launch_rmsnorm(x1, w->mlp_norm, h, rows, hidden, w->rms_eps, si.dtype, st);
    if (he != hipSuccess) return dev_fail("RMSNorm", he);
    for (long r0 = 0; r0 < rows; r0 += p.slab) {
        const long nr = rows - r0 < p.slab ? rows - r0 : p.slab;
        const char* hs = (const char*)h + (size_t)r0 * hidden * es;
        const char* xs = (const char*)x1 + (size_t)r0 * hidden * es;
        char* ys = (char*)y + (size_t)r0 * hidden * es;
        if (gemm_xwT(hs, hidden, w->w_gate_up, nullptr, gu, 2 * inter, nr, 2 * inter, hidden, si.dtype, st)) return fail(APE_ERR_DEVICE, "gate/up projection (rocBLAS) failed");
        he = launch_swiglu(gu, act, nr, inter, si.dtype, st);
        if (he != hipSuccess) return dev_fail("SiLU * up", he);
        if (gemm_xwT(act, inter, w->w_down, xs, ys, hidden, nr, hidden, inter, si.dtype, st)) return fail(APE_ERR_DEVICE, "down projection (rocBLAS) failed");
    }
    return APE_OK;
}

}  // namespace
}  // namespace ape

using namespace ape;

extern "C" {

size_t ape_layer_workspace_bytes(const ape_shape* shape, int32_t hidden, int32_t intermediate, int32_t total_rows) {
    ShapeInfo si;
    if (check_shape(shape, &si) != APE_OK) return 0;
    if (hidden < 8 || hidden % 8 || intermediate < 8 || intermediate % 8 || total_rows < 0) return 0;
    return plan_layer(si, hidden, intermediate, total_rows).total;
}

size_t ape_layers_workspace_bytes(const ape_shape* shape, int32_t hidden, int32_t intermediate, int32_t total_rows, int32_t n_layers) {
    ShapeInfo si;
    if (check_shape(shape, &si) != APE_OK) return 0;
    if (hidden < 8 || hidden % 8 || intermediate < 8 || intermediate % 8 || total_rows < 0 || n_layers < 1) return 0;
    const size_t es = si.dtype == APE_F32 ? 4 : 2;
    // one more [rows, hidden] buffer: the hidden states alternate between it and y
    return plan_layer(si, hidden, intermediate, total_rows).total + (n_layers > 1 ? align_up((size_t)total_rows * hidden * es, kWsAlign) : 0);
}

int ape_layer_encode(const ape_shape* shape, const ape_layer_weights* w, const void* x,
                     const void* k_prefix, const void* v_prefix, int32_t prefix_len,
                     const int32_t* cu_host, const int32_t* cu_dev, int32_t n_chunks,
                     void* k_cache, void* v_cache, void* y, const ape_layer_taps* taps,
                     void* workspace, size_t workspace_bytes, void* stream) {
    ShapeInfo si;
    int rc = check_shape(shape, &si);
    if (rc) return rc;
    rc = check_layer(w, 0);
    if (rc) return rc;
    if (prefix_len > 0 && (!k_prefix || !v_prefix)) return fail(APE_ERR_INVALID_ARG, "prefix KV is NULL");
    Contexts c;
    rc = check_contexts(si, prefix_len, cu_host, cu_dev, n_chunks, &c);
    if (rc) return rc;
    if (c.rows == 0) return APE_OK;
    if (!x || !y || !k_cache || !v_cache) return fail(APE_ERR_INVALID_ARG, "x, y, k_cache and v_cache must not be NULL");
    if (x == y) return fail(APE_ERR_INVALID_ARG, "y may not alias x");
    for (const void* p : {x, (const void*)y, (const void*)k_cache, (const void*)v_cache, k_prefix, v_prefix,
                          taps ? (const void*)taps->q_rot : nullptr, taps ? (const void*)taps->attn : nullptr})
        if (misaligned(p)) return fail(APE_ERR_INVALID_ARG, "data pointer %p is not 16-byte aligned", p);
    const LayerPlan p = plan_layer(si, w->hidden, w->intermediate, c.rows);
    if (!workspace || workspace_bytes < p.total)
        return fail(APE_ERR_WORKSPACE, "workspace of %zu bytes given, %zu needed (ape_layer_workspace_bytes gives the size)", workspace_bytes, p.total);
    if ((uintptr_t)workspace % kWsAlign) return fail(APE_ERR_WORKSPACE, "workspace must be %d-byte aligned", kWsAlign);
    hipStream_t st = (hipStream_t)stream;
    BlasCall lock;
    if (!blas_ready_for(st)) return fail(APE_ERR_DEVICE, "no rocBLAS handle for this device (under a graph capture the first call must come before the capture)");
    return run_layer(si, w, c, x, k_prefix, v_prefix, k_cache, v_cache, y, taps, (char*)workspace, p, st);
}

int ape_layers_encode(const ape_shape* shape, const ape_layer_weights* layers, int32_t n_layers, const void* x,
                      const void* const* k_prefix, const void* const* v_prefix, int32_t prefix_len,
                      const int32_t* cu_host, const int32_t* cu_dev, int32_t n_chunks,
                      void* const* k_cache, void* const* v_cache, void* y,
                      void* workspace, size_t workspace_bytes, void* stream) {
    ShapeInfo si;
    int rc = check_shape(shape, &si);
    if (rc) return rc;
    if (n_layers < 1) return fail(APE_ERR_INVALID_ARG, "n_layers %d < 1", n_layers);
    if (!layers) return fail(APE_ERR_INVALID_ARG, "layer weights are NULL");
    for (int l = 0; l < n_layers; ++l) {
        rc = check_layer(&layers[l], l);
        if (rc) return rc;
        if (layers[l].hidden != layers[0].hidden || layers[l].intermediate != layers[0].intermediate)
            return fail(APE_ERR_INVALID_ARG, "layer %d: every layer of a stack has the same hidden and intermediate width", l);
    }
    if (prefix_len > 0 && (!k_prefix || !v_prefix)) return fail(APE_ERR_INVALID_ARG, "prefix KV tables are NULL");
    Contexts c;
    rc = check_contexts(si, prefix_len, cu_host, cu_dev, n_chunks, &c);
    if (rc) return rc;
    if (c.rows == 0) return APE_OK;
    if (!x || !y || !k_cache || !v_cache) return fail(APE_ERR_INVALID_ARG, "x, y and the cache tables must not be NULL");
    if (x == y) return fail(APE_ERR_INVALID_ARG, "y may not alias x");
    if (misaligned(x) || misaligned(y)) return fail(APE_ERR_INVALID_ARG, "x and y must be 16-byte aligned");
    for (int l = 0; l < n_layers; ++l) {
        if (!k_cache[l] || !v_cache[l]) return fail(APE_ERR_INVALID_ARG, "layer %d: cache pointer is NULL", l);
        if (prefix_len > 0 && (!k_prefix[l] || !v_prefix[l])) return fail(APE_ERR_INVALID_ARG, "layer %d: prefix KV is NULL", l);
        for (const void* p : {(const void*)k_cache[l], (const void*)v_cache[l], prefix_len > 0 ? k_prefix[l] : nullptr, prefix_len > 0 ? v_prefix[l] : nullptr})
            if (misaligned(p)) return fail(APE_ERR_INVALID_ARG, "layer %d: data pointer %p is not 16-byte aligned", l, p);
    }
    const int hidden = layers[0].hidden, inter = layers[0].intermediate;
    const LayerPlan p = plan_layer(si, hidden, inter, c.rows);
    const size_t es = si.dtype == APE_F32 ? 4 : 2;
    const size_t need = p.total + (n_layers > 1 ? align_up((size_t)c.rows * hidden * es, kWsAlign) : 0);
    if (!workspace || workspace_bytes < need)
        return fail(APE_ERR_WORKSPACE, "workspace of %zu bytes given, %zu needed (ape_layers_workspace_bytes gives the size)", workspace_bytes, need);
    if ((uintptr_t)workspace % kWsAlign) return fail(APE_ERR_WORKSPACE, "workspace must be %d-byte aligned", kWsAlign);
    hipStream_t st = (hipStream_t)stream;
    BlasCall lock;
    if (!blas_ready_for(st)) return fail(APE_ERR_DEVICE, "no rocBLAS handle for this device (under a graph capture the first call must come before the capture)");
    // the hidden states alternate between y and the spare buffer so that the last layer writes y
    void* spare = (char*)workspace + p.total;
    const void* in = x;
    for (int l = 0; l < n_layers; ++l) {
        void* out = (n_layers - 1 - l) % 2 == 0 ? y : spare;
        rc = run_layer(si, &layers[l], c, in, prefix_len > 0 ? k_prefix[l] : nullptr, prefix_len > 0 ? v_prefix[l] : nullptr,
                       k_cache[l], v_cache[l], out, nullptr, (char*)workspace, p, st);
        if (rc) return rc;
        in = out;
    }
    return APE_OK;
}

}  // extern "C"
