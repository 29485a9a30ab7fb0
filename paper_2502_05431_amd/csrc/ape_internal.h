// Internal declarations shared by the host entry points and the gfx950 kernels.
// Not part of the public ABI (that is include/ape.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ape.h"

namespace ape {

// Device-visible copy of one ape_request (pointers are device pointers).
struct KvView {
    const void* k_prefix;
    const void* v_prefix;
    const void* const* k_chunks;
    const void* const* v_chunks;
    const int32_t* cu;          // [n_chunks + 1]
    const void* k_self;
    const void* v_self;
    int32_t prefix_len;
    int32_t n_chunks;
    int32_t total_ctx;
    int32_t self_len;
    float temperature;
    float scale;
};

constexpr int kMaxReqPerLaunch = 32;     // requests whose descriptors travel in one kernel-argument block
constexpr int kMaxSplits = 64;           // upper bound of context splits per (request, head)
constexpr int kWsAlign = 256;

// Kernel-argument block of the query-time kernels (prefill and decode).
struct QueryArgs {
    KvView req[kMaxReqPerLaunch];
    const void* q;              // [batch*q_len, Hq, d]
    float* part_o;              // [n_splits_total][units][d], unit = (request*q_len + row)*Hq + head
    float* part_lse;            // [n_splits_total][units]
    int32_t n_req;
    int32_t q_len;              // rows per request
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t n_ctx_splits;       // splits of the context group; split index n_ctx_splits is prefix + self
    int32_t ctx_split_len;      // context tokens per split (multiple of 64)
    const int32_t* split_ranges; // NULL: split s covers tokens [s*ctx_split_len, ...) of the pooled contexts.
                                // Else (one request only) DEVICE [2*n_ctx_splits]: split s covers tokens
                                // [split_ranges[2s], split_ranges[2s+1]) of the pooled contexts; empty if equal
    int32_t units_total;        // n_req * q_len * Hq (stride of the split dimension)
    int32_t req_base;           // index of req[0] in the whole batch
};

struct MergeArgs {
    const float* part_o;
    const float* part_lse;
    void* out;                  // [units][d], dtype
    float* lse_out;             // NULL or fp32
    float scale[kMaxReqPerLaunch];
    int32_t total_ctx[kMaxReqPerLaunch];   // context tokens of each request: splits past them were never written
    int32_t ctx_split_len;
    int32_t n_req;
    int32_t q_len;
    int32_t n_q_heads;
    int32_t head_dim;
    int32_t n_ctx_splits;
    int32_t n_splits_total;
    int32_t units_total;
    int32_t req_base;
    int32_t lse_head_major;     // 1: lse_out[h*q_len + r] (prefill); 0: lse_out[unit] (decode)
    int32_t dtype;
};

// Device-side plan of a tree call, written into the workspace by the plan kernel and read by the
// attention and merge kernels.  Every node whose children are contexts ("group") owns a run of
// consecutive splits that cover its contexts' tokens in runs of split_len; contexts of one group
// merge exactly (Appendix C.1), so no split ever needs to stop at a context boundary inside a group.
// Layout in int32 words: [0] number of splits in use, [1..3] unused, then first_split[n_nodes],
// n_splits[n_nodes] (0 for nodes whose children are nodes), split_ranges[2 * max_splits].
struct TreePlanLayout {
    int n_nodes, max_splits;
    __host__ __device__ long first_split_at() const { return 4; }
    __host__ __device__ long n_splits_at() const { return 4 + (long)n_nodes; }
    __host__ __device__ long ranges_at() const { return 4 + 2 * (long)n_nodes; }
    __host__ __device__ long words() const { return 4 + 2 * (long)n_nodes + 2 * (long)max_splits; }
};

struct TreePlanArgs {
    const ape_tree_node* nodes; // device [n_nodes]
    const int32_t* cu;          // device [n_chunks + 1]
    int32_t* plan;              // device, TreePlanLayout
    int32_t n_nodes;
    int32_t max_splits;
    int32_t split_len;
};

// Kernel-argument block of the tree merge (Appendix C.2 per node, C.5).
constexpr int kMaxTreeLevels = APE_TREE_MAX_DEPTH;
constexpr int kMaxTreeSplits = 8192;
struct TreeMergeArgs {
    const float* part_o;        // [max_splits + 1][units][d]; split max_splits is prefix + self
    const float* part_lse;
    void* out;
    float* lse_out;             // NULL or fp32 [Hq, q_len]
    const ape_tree_node* nodes; // device [n_nodes]
    const int32_t* plan;        // device, TreePlanLayout
    int32_t n_nodes;
    int32_t max_splits;
    int32_t units_total;        // q_len * Hq
    int32_t q_len;
    int32_t n_q_heads;
    int32_t head_dim;
    int32_t dtype;
    int32_t n_levels;
    int32_t level_start[kMaxTreeLevels + 1];   // nodes of level l: [level_start[l], level_start[l+1])
};

struct EncodeArgs {
    const void* q;              // packed [M, Hq, d]
    const void* k;              // packed [M, Hkv, d]
    const void* v;
    const void* k_prefix;
    const void* v_prefix;
    const int32_t* cu;          // device [n_chunks + 1]
    void* out;                  // packed [M, Hq, d]
    float* lse;                 // NULL or [Hq, M]
    int32_t n_chunks;
    int32_t prefix_len;
    int32_t total_rows;         // M
    int32_t max_chunk_len;
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t uniform_chunks;     // != 0: every chunk has max_chunk_len tokens (known on the host)
};

// Kernel-argument block of the rotary embedding + cache write.
struct RopeArgs {
    const void* q_raw;          // packed [M, Hq, d] or NULL
    const void* k_raw;          // packed [M, Hkv, d] or NULL
    const void* v_raw;          // packed [M, Hkv, d] or NULL
    void* q_rot;                // packed [M, Hq, d]
    void* const* k_cache;       // device [n_chunks] of device pointers [l_i, Hkv, d], or NULL with k_packed set
    void* const* v_cache;
    void* k_packed;             // alternative destination: one packed buffer [M, Hkv, d]
    void* v_packed;
    int64_t q_stride, k_stride, v_stride;   // elements between consecutive tokens of the raw inputs
    const int32_t* cu;          // device [n_chunks + 1]
    int32_t n_chunks;
    int32_t total_rows;         // M
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t head_dim;           // even, <= 256
    int32_t position_offset;    // position of the first token of every segment
    double inv_freq[128];       // base^(-2c/d), c < d/2, computed on the host in double
};

#if defined(__HIPCC__)
// Field access into the kernel-argument segment.  A by-value argument struct that is indexed
// with a run-time index would be copied to scratch as a whole; reading it through the
// segment pointer keeps the accesses scalar loads.  Valid only for kernels whose FIRST
// argument is the struct in question (it then starts at offset 0 of the segment).
template <typename Args>
__device__ __forceinline__ __attribute__((address_space(4))) const Args* kernarg() {
    return (__attribute__((address_space(4))) const Args*)__builtin_amdgcn_kernarg_segment_ptr();
}

// The chunk tables (pointer arrays, cu_chunk_lens) are read-only for the whole launch and are
// indexed with wavefront-uniform indices.  They are read with explicit SCALAR loads: the results
// stay in scalar registers (uniform control flow around the block walkers) and, being counted by
// lgkmcnt, the reads do not drain the vector-memory queue that holds the K/V loads in flight
// (a vector load of a table entry would be followed by s_waitcnt vmcnt(0)).
// The address must be wavefront-uniform; the compiler moves it to scalar registers.
__device__ __forceinline__ uint64_t uniform_address(const void* p) {
    const uint64_t a = (uint64_t)p;
    // the builtin returns a signed int: go through uint32_t, or the low half would be sign-extended
    // into the high half
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)a);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32));
    return ((uint64_t)hi << 32) | (uint64_t)lo;
}
__device__ __forceinline__ int32_t scalar_load_i32(const int32_t* p) {
    int32_t v;
    asm volatile("s_load_dword %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(uniform_address(p)) : "memory");
    return v;
}
__device__ __forceinline__ const void* scalar_load_ptr(const void* const* p) {
    uint64_t v;
    asm volatile("s_load_dwordx2 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(uniform_address(p)) : "memory");
    return (const void*)v;
}

// The chunk that holds pooled context index t: the largest c in [0, n_chunks - 1] with cu[c] <= t
// (cu non-decreasing, cu[0] = 0 <= t; n_chunks >= 1; t wavefront-uniform).  A binary search is a chain of
// log2(n) dependent loads, ~0.5 us each, in front of a workgroup's first K/V load; here the 64 lanes
// probe 64 evenly spaced entries at once and a ballot narrows the range 64-fold per round trip: one
// round for up to 64 chunks, two for up to 4096.
__device__ __forceinline__ int find_chunk(const int32_t* cu, int n_chunks, int t) {
    const int lane = threadIdx.x & 63;
    int lo = 0, hi = n_chunks - 1;                                     // cu[lo] <= t holds throughout; the answer is <= hi
    while (lo < hi) {
        const int step = (hi - lo + 63) >> 6;                          // >= 1; lane 63 probes hi
        const int idx = min(lo + (lane + 1) * step, hi);               // non-decreasing over the lanes
        const int cnt = __builtin_popcountll(__builtin_amdgcn_ballot_w64(cu[idx] <= t));   // true for a prefix of the lanes
        if (cnt == 64) { lo = hi; break; }
        const int first_false = min(lo + (cnt + 1) * step, hi);        // lane cnt's probe: the answer lies before it
        if (cnt > 0) lo = min(lo + cnt * step, hi);                    // lane cnt-1's probe (a smaller index than lane cnt's)
        hi = first_false - 1;
    }
    return __builtin_amdgcn_readfirstlane(lo);
}

// Context tokens [t0, t1) (indices into the pooled contexts) that split `split` of request view
// `kv` covers; t0 >= t1 for an empty split.  `split` must be wavefront-uniform.
__device__ __forceinline__ void ctx_split_range(const QueryArgs& a, const KvView& kv, int split, long& t0, long& t1) {
    if (a.split_ranges == nullptr) {
        t0 = (long)split * a.ctx_split_len;
        t1 = min((long)kv.total_ctx, t0 + a.ctx_split_len);
        return;
    }
    t0 = scalar_load_i32(a.split_ranges + 2 * split);
    t1 = scalar_load_i32(a.split_ranges + 2 * split + 1);
}

// One chunk-table entry in a single round trip: cu[c + 1] and the K and V base pointers of chunk c
// (three scalar loads issued back to back, one wait).
__device__ __forceinline__ void scalar_load_chunk(const int32_t* cu_next, const void* const* kp, const void* const* vp,
                                                  int32_t& c1, const void*& k, const void*& v) {
    uint64_t kk, vv;
    asm volatile("s_load_dword %0, %3, 0x0\n\ts_load_dwordx2 %1, %4, 0x0\n\ts_load_dwordx2 %2, %5, 0x0\n\ts_waitcnt lgkmcnt(0)"
                 : "=&s"(c1), "=&s"(kk), "=&s"(vv)
                 : "s"(uniform_address(cu_next)), "s"(uniform_address(kp)), "s"(uniform_address(vp)) : "memory");
    k = (const void*)kk; v = (const void*)vv;
}

template <typename Args>
__device__ __forceinline__ KvView load_view(int rq) {
    auto ap = kernarg<Args>();
    KvView v;
    v.k_prefix = ap->req[rq].k_prefix; v.v_prefix = ap->req[rq].v_prefix;
    v.k_chunks = ap->req[rq].k_chunks; v.v_chunks = ap->req[rq].v_chunks; v.cu = ap->req[rq].cu;
    v.k_self = ap->req[rq].k_self; v.v_self = ap->req[rq].v_self;
    v.prefix_len = ap->req[rq].prefix_len; v.n_chunks = ap->req[rq].n_chunks;
    v.total_ctx = ap->req[rq].total_ctx; v.self_len = ap->req[rq].self_len;
    v.temperature = ap->req[rq].temperature; v.scale = ap->req[rq].scale;
    return v;
}
#endif

// ---- host helpers of the entry points (defined in ape_api.hip; the layer library, a separate
// shared object, links against them) --------------------------------------------------------
struct ShapeInfo {
    int hq, hkv, d, dtype, group;
    bool force_generic;
    bool mfma;                  // matrix-core kernels cover this shape
};
// records the text ape_last_error() returns on this thread, returns `code`
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
int check_shape(const ape_shape* s, ShapeInfo* o);
// size limits of an encode launch (see the header's general conventions)
int check_encode_size(const ShapeInfo& si, int n_chunks, int max_len, long total_rows);

// Split plan shared by ape_workspace_bytes and the launches.
struct QueryPlan {
    int n_ctx_splits;
    int ctx_split_len;
    int n_splits_total;
    int n_bound;           // >= n_ctx_splits of this plan and of the plan for any shorter context with the same base and target
    int block_rows;        // query tile of the flash prefill this plan was made for (0: not a flash prefill)
};

// ---- launchers (each returns hipGetLastError() of its launch) ------------------------------
hipError_t launch_generic_query(const QueryArgs& a, int dtype, hipStream_t s);
hipError_t launch_generic_encode(const EncodeArgs& a, int dtype, hipStream_t s);
hipError_t launch_merge(const MergeArgs& a, hipStream_t s);
hipError_t launch_rope_write(const RopeArgs& a, int dtype, hipStream_t s);
hipError_t launch_tree_plan(const TreePlanArgs& a, hipStream_t s);
hipError_t launch_tree_merge(const TreeMergeArgs& a, hipStream_t s);
hipError_t launch_flash_prefill(const QueryArgs& a, int block_rows, hipStream_t s);     // bf16, d = 128; block_rows from the plan
hipError_t launch_flash_encode(const EncodeArgs& a, hipStream_t s);     // bf16, d = 128

// rows of (token, group-head) pairs one flash workgroup covers for a given amount of rows
int flash_block_rows(int rows_per_kv_head);
// the same for the query prefill, which also looks at the context length (see the definition), and
// the number of workgroups its split plan aims at
int flash_prefill_block_rows(int rows_per_kv_head, long max_ctx);
int flash_prefill_target_workgroups(int rows_per_kv_head, long max_ctx);
// the context lengths at which those two change their answer (each holds up to and including its value):
// one narrow workgroup per CU, then two, then the wide tile -- the sooner the more query rows there are
constexpr long kPrefillOneWorkgroupPerCuMaxCtx = 12288;
long flash_prefill_narrow_tile_max_ctx(int rows_per_kv_head);

}  // namespace ape
