// Generic gfx950 kernels of the APE attention path: any head_dim <= 256, fp32 or bf16 storage,
// fp32 arithmetic on the vector ALUs.  They serve the fp32 workload and every shape the
// matrix-core kernels do not cover.  One wavefront (64 lanes) owns one (query row, query head)
// and one split of its keys; the split-merge kernel at the end of this file is shared with the
// matrix-core kernels.
//
// Math (arXiv 2502.05431): Section 4.4 refined attention in the block form of Appendix C --
// each block yields a softmax-weighted value vector and a LogSumExp (C.1); the context blocks
// use scores q.k/(T sqrt d); the merge multiplies the pooled context LogSumExp by S (C.3/C.4).
#include "ape_internal.h"

#include <math.h>

namespace ape {
namespace {

constexpr int kWave = 64;
constexpr int kMaxDimRegs = 4;          // head_dim <= 256

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(__bf16 x) { return (float)x; }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// Running state of one wavefront's online softmax (natural-log units).
struct State {
    float m;                       // running maximum of the scaled scores
    float l;                       // running sum of exp(score - m)
    float acc[kMaxDimRegs];        // lane owns dims lane + 64*k
};

// Attend to n consecutive tokens of one KV head: K/V rows at k + j*stride, v + j*stride.
// q_lds holds the query vector in fp32.  `scale` multiplies q.k.
template <typename T>
__device__ __forceinline__ void attend_rows(const T* __restrict__ k, const T* __restrict__ v, long stride, int n,
                                            int d, float scale, const float* q_lds, State& st) {
    const int lane = threadIdx.x & (kWave - 1);
    for (int j0 = 0; j0 < n; j0 += kWave) {
        const int j = j0 + lane;
        const bool valid = j < n;
        float s = -INFINITY;
        if (valid) {
            const T* kr = k + (long)j * stride;
            float dot = 0.f;
            for (int c = 0; c < d; ++c) dot = fmaf(q_lds[c], to_f32(kr[c]), dot);
            s = dot * scale;
        }
        const float m_new = fmaxf(st.m, wave_max(s));          // finite: at least lane 0 is valid
        const float p = valid ? expf(s - m_new) : 0.f;
        const float alpha = expf(st.m - m_new);                // exp(-inf) = 0 on the first block
        st.l = st.l * alpha + wave_sum(p);
        st.m = m_new;
#pragma unroll
        for (int r = 0; r < kMaxDimRegs; ++r) st.acc[r] *= alpha;
        const int cnt = min(kWave, n - j0);
        for (int jj = 0; jj < cnt; ++jj) {
            const float pj = __shfl(p, jj);
            const T* vr = v + (long)(j0 + jj) * stride;
#pragma unroll
            for (int r = 0; r < kMaxDimRegs; ++r) {
                const int c = lane + kWave * r;
                if (c < d) st.acc[r] = fmaf(pj, to_f32(vr[c]), st.acc[r]);
            }
        }
    }
}

// Block result (Appendix C.1): o = softmax-weighted values, lse = LogSumExp; empty block: 0, -inf.
__device__ __forceinline__ void store_block(const State& st, int d, float* o, float* lse) {
    const int lane = threadIdx.x & (kWave - 1);
    const float inv = st.l > 0.f ? 1.f / st.l : 0.f;
#pragma unroll
    for (int r = 0; r < kMaxDimRegs; ++r) {
        const int c = lane + kWave * r;
        if (c < d) o[c] = st.acc[r] * inv;
    }
    if (lane == 0) *lse = st.l > 0.f ? st.m + logf(st.l) : -INFINITY;
}

// grid: x = (request*q_len + row)*Hq + head, y = split (n_ctx_splits context splits, then prefix+self)
template <typename T>
__global__ __launch_bounds__(kWave) void generic_query_kernel(const QueryArgs a) {
    __shared__ float q_lds[256];
    const int lane = threadIdx.x;
    const int unit = blockIdx.x;
    const int split = blockIdx.y;
    const int d = a.head_dim, hq = a.n_q_heads;
    const int h = unit % hq;
    const int row = (unit / hq) % a.q_len;
    const int rq = unit / (hq * a.q_len);
    const KvView kv = load_view<QueryArgs>(rq);      // scalar loads from the kernel-argument segment
    const int hk = h / (hq / a.n_kv_heads);
    const long stride = (long)a.n_kv_heads * d;

    const T* qv = (const T*)a.q + (long)unit * d;
    for (int c = lane; c < d; c += kWave) q_lds[c] = to_f32(qv[c]);
    __syncthreads();

    State st;
    st.m = -INFINITY; st.l = 0.f;
#pragma unroll
    for (int r = 0; r < kMaxDimRegs; ++r) st.acc[r] = 0.f;
    const float inv_sqrt_d = rsqrtf((float)d);

    if (split < a.n_ctx_splits) {
        // context group, tokens [t0, t1) of the pooled contexts, temperature in the scale
        const float scale = inv_sqrt_d / kv.temperature;
        long t0, t1;
        ctx_split_range(a, kv, split, t0, t1);
        if (t0 < t1) {
            int c = 0;                                   // chunk that holds t0 (upper-bound search)
            int lo = 0, hi = kv.n_chunks - 1;
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (kv.cu[mid] <= t0) lo = mid; else hi = mid - 1;
            }
            c = lo;
            while (t0 < t1 && c < kv.n_chunks) {
                const long c0 = kv.cu[c], c1 = kv.cu[c + 1];
                const long e = min(c1, t1);
                if (e > t0) {
                    const T* kc = (const T*)kv.k_chunks[c] + (t0 - c0) * stride + (long)hk * d;
                    const T* vc = (const T*)kv.v_chunks[c] + (t0 - c0) * stride + (long)hk * d;
                    attend_rows<T>(kc, vc, stride, (int)(e - t0), d, scale, q_lds, st);
                    t0 = e;
                }
                ++c;
            }
        }
    } else {
        // non-context group: whole prefix, then the causal part of the self KV
        if (kv.prefix_len > 0)
            attend_rows<T>((const T*)kv.k_prefix + (long)hk * d, (const T*)kv.v_prefix + (long)hk * d, stride,
                           kv.prefix_len, d, inv_sqrt_d, q_lds, st);
        const int n_self = kv.self_len - a.q_len + row + 1;
        attend_rows<T>((const T*)kv.k_self + (long)hk * d, (const T*)kv.v_self + (long)hk * d, stride,
                       n_self, d, inv_sqrt_d, q_lds, st);
    }
    const long gunit = (long)a.req_base * a.q_len * hq + unit;
    const long slot = (long)split * a.units_total + gunit;
    store_block(st, d, a.part_o + slot * d, a.part_lse + slot);
}

// grid: x = packed row * Hq + head.  Writes the final output (no splits).
template <typename T>
__global__ __launch_bounds__(kWave) void generic_encode_kernel(const EncodeArgs a) {
    __shared__ float q_lds[256];
    __shared__ float o_lds[256];
    __shared__ float lse_lds;
    const int lane = threadIdx.x;
    const long unit = blockIdx.x;
    const int d = a.head_dim, hq = a.n_q_heads;
    const int h = (int)(unit % hq);
    const int row = (int)(unit / hq);
    const int hk = h / (hq / a.n_kv_heads);
    const long stride = (long)a.n_kv_heads * d;

    int c0 = 0;                                         // first packed row of the chunk that owns `row`
    if (a.cu) {                                         // cu == NULL: a single chunk starting at row 0
        int lo = 0, hi = a.n_chunks - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (a.cu[mid] <= row) lo = mid; else hi = mid - 1;
        }
        c0 = a.cu[lo];
    }

    const T* qv = (const T*)a.q + unit * d;
    for (int c = lane; c < d; c += kWave) q_lds[c] = to_f32(qv[c]);
    __syncthreads();

    State st;
    st.m = -INFINITY; st.l = 0.f;
#pragma unroll
    for (int r = 0; r < kMaxDimRegs; ++r) st.acc[r] = 0.f;
    const float inv_sqrt_d = rsqrtf((float)d);
    if (a.prefix_len > 0)
        attend_rows<T>((const T*)a.k_prefix + (long)hk * d, (const T*)a.v_prefix + (long)hk * d, stride,
                       a.prefix_len, d, inv_sqrt_d, q_lds, st);
    attend_rows<T>((const T*)a.k + (long)c0 * stride + (long)hk * d, (const T*)a.v + (long)c0 * stride + (long)hk * d,
                   stride, row - c0 + 1, d, inv_sqrt_d, q_lds, st);
    store_block(st, d, o_lds, &lse_lds);
    __syncthreads();
    T* o = (T*)a.out + unit * d;
    for (int c = lane; c < d; c += kWave) o[c] = (T)o_lds[c];
    if (a.lse && lane == 0) a.lse[(long)h * a.total_rows + row] = lse_lds;
}

// Merge of the split results (Appendix C.1 for splits of one group, C.3/C.4 across the two
// groups): the context splits are merged first, exactly; only then is the pooled context
// LogSumExp multiplied by S -- (sum of splits)^S is not the sum of the splits^S.
// grid: x = unit; a workgroup of kMergeWaves wavefronts per unit.  Every wavefront computes the
// split weights (one coalesced read of the LogSumExps, a wavefront reduction); the wavefronts
// then share out the splits, each accumulating its weighted rows with several loads in flight,
// and are combined through LDS.  (A serial loop over 64 splits cost 61 us at batch 1.)
constexpr int kMergeWaves = 4;
constexpr int kMergeWavesFew = 16;

// One group of splits [s0, s1): this wavefront's share of sum_s w_s o_s into acc (lane owns dims
// lane + 64 r), with w_s = exp(lse_s - max); returns the group's max and sum of weights.
template <int W>
__device__ __forceinline__ void merge_group(const MergeArgs& a, long gunit, int s0, int s1, int wave, int lane,
                                            float (&acc)[kMaxDimRegs], float& m_out, float& z_out) {
    const int d = a.head_dim;
    float m = -INFINITY;
    for (int s = s0 + lane; s < s1; s += kWave) m = fmaxf(m, a.part_lse[(long)s * a.units_total + gunit]);
    m = wave_max(m);
    float z = 0.f;
    if (m > -INFINITY) {
        for (int c0 = s0; c0 < s1; c0 += kWave) {                   // chunks of 64 splits: lane <-> split
            const int s_mine = c0 + lane;
            const float w_mine = s_mine < s1 ? expf(a.part_lse[(long)s_mine * a.units_total + gunit] - m) : 0.f;   // 0 for empty splits
            z += w_mine;
            const int cnt = min(kWave, s1 - c0);
            constexpr int UN = 4;                                       // rows in flight per wavefront
            for (int i = wave; i < cnt; i += UN * W) {
                float w[UN], v[UN][kMaxDimRegs];
#pragma unroll
                for (int u = 0; u < UN; ++u) {
                    const int ii = i + u * W;
                    w[u] = ii < cnt ? __shfl(w_mine, min(ii, kWave - 1)) : 0.f;
                    const float* o = a.part_o + ((long)(c0 + min(ii, cnt - 1)) * a.units_total + gunit) * d;
#pragma unroll
                    for (int r = 0; r < kMaxDimRegs; ++r) {
                        const int c = lane + kWave * r;
                        v[u][r] = c < d ? o[c] : 0.f;
                    }
                }
#pragma unroll
                for (int u = 0; u < UN; ++u)
#pragma unroll
                    for (int r = 0; r < kMaxDimRegs; ++r) acc[r] = fmaf(w[u], v[u][r], acc[r]);
            }
        }
        z = wave_sum(z);
    }
    m_out = m; z_out = z;
}

// W wavefronts per unit: kMergeWaves when there are many units (the launch is then bound by its
// traffic), kMergeWavesFew for a few units with many splits each (decode of a long context at a small
// batch: 32 units x 64 splits), where the time is a chain of round trips and W x 4 rows in flight
// cover all splits in one of them.
template <typename T, int W>
__global__ __launch_bounds__(kWave * W) void merge_kernel(const MergeArgs a) {
    __shared__ float part[2][W][kWave * kMaxDimRegs];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int unit = blockIdx.x;                                    // within this launch
    const int d = a.head_dim, hq = a.n_q_heads;
    const int rq = unit / (hq * a.q_len);
    const long gunit = (long)a.req_base * a.q_len * hq + unit;
    const float S = kernarg<MergeArgs>()->scale[rq];

    float acc_c[kMaxDimRegs], acc_o[kMaxDimRegs];
#pragma unroll
    for (int r = 0; r < kMaxDimRegs; ++r) { acc_c[r] = 0.f; acc_o[r] = 0.f; }
    float mc, zc, mo, zo;
    // context group: only the splits that hold tokens of THIS request (a shorter context in a
    // batch leaves the trailing splits untouched)
    const int tc = kernarg<MergeArgs>()->total_ctx[rq];
    const int n_ctx = min(a.n_ctx_splits, (tc + a.ctx_split_len - 1) / a.ctx_split_len);
    merge_group<W>(a, gunit, 0, n_ctx, wave, lane, acc_c, mc, zc);
    merge_group<W>(a, gunit, a.n_ctx_splits, a.n_splits_total, wave, lane, acc_o, mo, zo);   // prefix + self: never empty
#pragma unroll
    for (int r = 0; r < kMaxDimRegs; ++r) {
        part[0][wave][lane + kWave * r] = acc_c[r];
        part[1][wave][lane + kWave * r] = acc_o[r];
    }
    __syncthreads();
    if (wave != 0) return;
#pragma unroll
    for (int r = 0; r < kMaxDimRegs; ++r) {
        acc_c[r] = 0.f; acc_o[r] = 0.f;
#pragma unroll
        for (int w = 0; w < W; ++w) { acc_c[r] += part[0][w][lane + kWave * r]; acc_o[r] += part[1][w][lane + kWave * r]; }
    }
    const float lse_c = mc > -INFINITY ? mc + logf(zc) : -INFINITY;   // log Z_ctx
    const float inv_zc = zc > 0.f ? 1.f / zc : 0.f;
    const float lse_o = mo + logf(zo);
    const float inv_zo = 1.f / zo;

    // softmax over (S * lse_c, lse_o)
    const float ac = lse_c > -INFINITY ? S * lse_c : -INFINITY;
    const float mx = fmaxf(ac, lse_o);
    const float ec = expf(ac - mx), eo = expf(lse_o - mx);
    const float wc = ec / (ec + eo), wo = eo / (ec + eo);

    T* out = (T*)a.out + gunit * d;
#pragma unroll
    for (int r = 0; r < kMaxDimRegs; ++r) {
        const int c = lane + kWave * r;
        if (c < d) out[c] = (T)(wc * acc_c[r] * inv_zc + wo * acc_o[r] * inv_zo);
    }
    if (a.lse_out && lane == 0) {
        const float lse = mx + logf(ec + eo);
        if (a.lse_head_major) {                                     // [request, head, row]
            const int h = unit % hq, row = (unit / hq) % a.q_len;
            a.lse_out[((long)(a.req_base + rq) * hq + h) * a.q_len + row] = lse;
        } else {
            a.lse_out[gunit] = lse;
        }
    }
}

// The same merge for MANY units of head_dim 128 (a query prefill: 8192 units of 9 splits; a batched
// decode step): a workgroup per unit spends its time being launched (8192 workgroups took 25 us for
// 40 MB).  Here half a wavefront owns a unit -- lane j holds dims 4j .. 4j+3, so a split's row is one
// 16-byte load per lane -- eight units per workgroup, no LDS and no barrier: one round trip for the
// LogSumExps (lane j reads splits j, j + 32, j + 64), the weights by half-wavefront reductions, then
// the rows with eight loads in flight.
constexpr int kMergeUnitsPerBlock = 8;
template <typename T>
__global__ __launch_bounds__(256) void merge_units_kernel(const MergeArgs a) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int half = lane >> 5, j = lane & 31;
    const long n_units = (long)a.n_req * a.q_len * a.n_q_heads;
    const long unit_raw = ((long)blockIdx.x * 4 + wave) * 2 + half;
    const bool valid = unit_raw < n_units;
    const long unit = valid ? unit_raw : n_units - 1;                // (a spare half-wavefront recomputes the last unit and stores nothing)
    const int hq = a.n_q_heads;
    const int rq = (int)(unit / ((long)hq * a.q_len));
    const long gunit = (long)a.req_base * a.q_len * hq + unit;
    auto ka = kernarg<MergeArgs>();
    const float S = ka->scale[rq];                                   // (per lane: the two halves may belong to different requests)
    const int tc = ka->total_ctx[rq];
    const int n_split = a.n_ctx_splits;                              // slots of the context group; slot n_split is prefix + self
    const int n_ctx = min(n_split, (tc + a.ctx_split_len - 1) / a.ctx_split_len);   // those this request wrote
    // LogSumExps: slot s lives in lane s % 32 of this half, register s / 32 (at most 65 slots)
    float l[3];
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int sl = j + 32 * r;
        const bool used = sl < n_ctx || sl == n_split;
        l[r] = used ? a.part_lse[(long)sl * a.units_total + gunit] : -INFINITY;
    }
    auto half_max = [](float x) {
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
        return x;
    };
    auto half_sum = [](float x) {
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) x += __shfl_xor(x, o);
        return x;
    };
    float lc[3];                                                     // context slots only
#pragma unroll
    for (int r = 0; r < 3; ++r) lc[r] = (j + 32 * r) < n_ctx ? l[r] : -INFINITY;
    const float mc = half_max(fmaxf(fmaxf(lc[0], lc[1]), lc[2]));
    float e[3];
#pragma unroll
    for (int r = 0; r < 3; ++r) e[r] = mc > -INFINITY ? expf(lc[r] - mc) : 0.f;   // 0 for empty and unused slots
    const float zc = half_sum(e[0] + e[1] + e[2]);
    const float lse_o = __shfl(l[n_split >> 5], (n_split & 31) + 32 * half);       // prefix + self: never empty
    // the context splits are pooled first; only then is their LogSumExp multiplied by S
    const float lse_c = zc > 0.f ? mc + logf(zc) : -INFINITY;
    const float ac = lse_c > -INFINITY ? S * lse_c : -INFINITY;
    const float mx = fmaxf(ac, lse_o);
    const float ec = expf(ac - mx), eo = expf(lse_o - mx);
    const float wc = ec / (ec + eo), wo = eo / (ec + eo);
    float w[3];                                                      // weight of this lane's slots in the output
#pragma unroll
    for (int r = 0; r < 3; ++r) w[r] = (j + 32 * r) == n_split ? wo : (zc > 0.f ? wc * e[r] / zc : 0.f);

    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    const float* base = a.part_o + gunit * 128 + 4 * j;
    const long slot_stride = (long)a.units_total * 128;
    const int n_slots = n_split + 1;                                 // wavefront-uniform loop bound
    constexpr int UN = 8;
    for (int s0 = 0; s0 < n_slots; s0 += UN) {
        float4 v[UN];
        float ws[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int sl = min(s0 + u, n_slots - 1);
            const float wl = __shfl(sl < 32 ? w[0] : sl < 64 ? w[1] : w[2], (sl & 31) + 32 * half);
            ws[u] = s0 + u < n_slots ? wl : 0.f;
            // a slot this request did not write is never read (its weight is 0; read the prefix + self slot instead)
            const int src = (sl < n_ctx || sl == n_split) ? sl : n_split;
            v[u] = *(const float4*)(base + src * slot_stride);
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            acc.x = fmaf(ws[u], v[u].x, acc.x); acc.y = fmaf(ws[u], v[u].y, acc.y);
            acc.z = fmaf(ws[u], v[u].z, acc.z); acc.w = fmaf(ws[u], v[u].w, acc.w);
        }
    }
    if (!valid) return;
    T* out = (T*)a.out + gunit * 128 + 4 * j;
    if constexpr (sizeof(T) == 4) {
        *(float4*)out = acc;
    } else {
        const T o4[4] = {(T)acc.x, (T)acc.y, (T)acc.z, (T)acc.w};
        *(uint2*)out = *(const uint2*)o4;
    }
    if (a.lse_out && j == 0) {
        const float lse = mx + logf(ec + eo);
        if (a.lse_head_major) {                                     // [request, head, row]
            const int h = (int)(unit % hq), row = (int)((unit / hq) % a.q_len);
            a.lse_out[((long)(a.req_base + rq) * hq + h) * a.q_len + row] = lse;
        } else {
            a.lse_out[gunit] = lse;
        }
    }
}

// ------------------------------------------------------------------------------------------
// Tree of contexts (Appendix C.2 applied at every node, Appendix C.5).
//
// Plan kernel: one workgroup.  A node whose children are contexts owns the tokens
// [cu[first], cu[first + count]) of the pooled contexts (contexts of one node merge exactly,
// Appendix C.1, so they need no boundary between them) and gets ceil(tokens / split_len) splits.
// An exclusive scan over the nodes gives every such node its first split; the ranges of the
// splits in use are written out, the slots behind them are left empty.
constexpr int kPlanThreads = 1024;
__global__ __launch_bounds__(kPlanThreads) void tree_plan_kernel(const TreePlanArgs a) {
    __shared__ int cnt[APE_TREE_MAX_NODES];
    __shared__ int off[APE_TREE_MAX_NODES];
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const TreePlanLayout lay{a.n_nodes, a.max_splits};
    int32_t* first_split = a.plan + lay.first_split_at();
    int32_t* n_splits = a.plan + lay.n_splits_at();
    int32_t* ranges = a.plan + lay.ranges_at();
    for (int i = tid; i < 2 * a.max_splits; i += kPlanThreads) ranges[i] = 0;
    for (int n = tid; n < APE_TREE_MAX_NODES; n += kPlanThreads) {
        int c = 0;
        if (n < a.n_nodes) {
            const ape_tree_node me = a.nodes[n];
            if (me.leaf_children) c = (a.cu[me.first + me.count] - a.cu[me.first] + a.split_len - 1) / a.split_len;
        }
        cnt[n] = c;
    }
    __syncthreads();
    if (tid < kWave) {
        // lane owns a run of consecutive nodes; wavefront scan of the run sums, then the runs
        constexpr int RUN = APE_TREE_MAX_NODES / kWave;
        int sum = 0;
        for (int j = 0; j < RUN; ++j) sum += cnt[lane * RUN + j];
        int incl = sum;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const int v = __shfl_up(incl, o);
            if (lane >= o) incl += v;
        }
        int run = incl - sum;
        for (int j = 0; j < RUN; ++j) { off[lane * RUN + j] = run; run += cnt[lane * RUN + j]; }
        if (lane == kWave - 1) a.plan[0] = min(incl, a.max_splits);
    }
    __syncthreads();
    for (int n = tid; n < a.n_nodes; n += kPlanThreads) {
        first_split[n] = off[n];
        n_splits[n] = cnt[n];
        if (cnt[n] > 0) {
            const ape_tree_node me = a.nodes[n];
            const int t_begin = a.cu[me.first], t_end = a.cu[me.first + me.count];
            for (int j = 0; j < cnt[n]; ++j) {
                const int s = off[n] + j;
                if (s >= a.max_splits) break;              // cannot happen with the host's bound; stay in bounds
                const int t0 = t_begin + j * a.split_len;
                ranges[2 * s] = t0;
                ranges[2 * s + 1] = min(t_end, t0 + a.split_len);
            }
        }
    }
}

// Tree merge.  One workgroup of kMergeWaves wavefronts per (row, head), everything in log units:
//   1. bottom-up, one level of nodes at a time, deepest first:
//        L_n = LogSumExp over the children of their values A; a child that is a split (of a node
//        whose children are contexts: exact merge, C.1) has A = its LogSumExp, a child node has
//        A = S_child L_child
//   2. the root meets the prefix+self block: Ltot = log(exp(S_root L_root) + exp(L_other)); top-down,
//      the log-weight of a child is W_child = W_n + A_child - L_n, starting at W_root = S_root L_root - Ltot
//   3. the output is the sum over splits of exp(W_split) o_split plus the prefix+self block with
//      weight exp(L_other - Ltot): the weights sum to one, nothing is divided.
// A level with many nodes gives each thread a node (children read serially); a narrow level
// gives each wavefront a node (children across the lanes).
struct TreeLds {
    const ape_tree_node* nd;
    const int* first_split;
    const float* node_l;
    const float* split_v;
};
__device__ __forceinline__ int child_count(const TreeLds& t, const int* n_splits, int n) {
    return t.nd[n].leaf_children ? n_splits[n] : t.nd[n].count;
}
__device__ __forceinline__ float child_value(const TreeLds& t, int n, int i) {
    if (t.nd[n].leaf_children) return t.split_v[t.first_split[n] + i];
    const int c = t.nd[n].first + i;
    return t.nd[c].scale * t.node_l[c];                   // S > 0: -inf stays -inf
}

template <typename T>
__global__ __launch_bounds__(kWave * kMergeWaves) void tree_merge_kernel(const TreeMergeArgs a) {
    extern __shared__ __attribute__((aligned(16))) char tree_lds[];
    __shared__ float part[kMergeWaves][kWave * kMaxDimRegs];
    __shared__ float s_ltot;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    constexpr int NT = kWave * kMergeWaves;
    const int unit = blockIdx.x;
    const int d = a.head_dim, U = a.units_total, n_nodes = a.n_nodes;
    const TreePlanLayout lay{a.n_nodes, a.max_splits};
    const int n_used = a.plan[0];

    ape_tree_node* nd = (ape_tree_node*)tree_lds;                  // [n_nodes]
    float* node_l = (float*)(nd + n_nodes);                        // [n_nodes] LogSumExp of the children's values
    float* node_w = node_l + n_nodes;                              // [n_nodes] log-weight in the result
    int* first_split = (int*)(node_w + n_nodes);                   // [n_nodes]
    int* n_splits = first_split + n_nodes;                         // [n_nodes]
    float* split_v = (float*)(n_splits + n_nodes);                 // [max_splits] LogSumExp, later log-weight

    for (int n = tid; n < n_nodes; n += NT) {
        nd[n] = a.nodes[n];
        first_split[n] = a.plan[lay.first_split_at() + n];
        n_splits[n] = a.plan[lay.n_splits_at() + n];
    }
    for (int s = tid; s < n_used; s += NT) split_v[s] = a.part_lse[(long)s * U + unit];
    const float l_other = a.part_lse[(long)a.max_splits * U + unit];
    __syncthreads();
    const TreeLds t{nd, first_split, node_l, split_v};

    // ---- bottom-up
    for (int lv = a.n_levels - 1; lv >= 0; --lv) {
        const int n0 = kernarg<TreeMergeArgs>()->level_start[lv], n1 = kernarg<TreeMergeArgs>()->level_start[lv + 1];
        if (n1 - n0 >= kWave) {
            for (int n = n0 + tid; n < n1; n += NT) {
                const int cn = child_count(t, n_splits, n);
                float m = -INFINITY;
                for (int i = 0; i < cn; ++i) m = fmaxf(m, child_value(t, n, i));
                float z = 0.f;
                if (m > -INFINITY)
                    for (int i = 0; i < cn; ++i) z += expf(child_value(t, n, i) - m);
                node_l[n] = m > -INFINITY ? m + logf(z) : -INFINITY;
            }
        } else {
            for (int n = n0 + wave; n < n1; n += kMergeWaves) {
                const int cn = child_count(t, n_splits, n);
                float m = -INFINITY;
                for (int i = lane; i < cn; i += kWave) m = fmaxf(m, child_value(t, n, i));
                m = wave_max(m);
                float z = 0.f;
                if (m > -INFINITY)
                    for (int i = lane; i < cn; i += kWave) z += expf(child_value(t, n, i) - m);
                z = wave_sum(z);
                if (lane == 0) node_l[n] = m > -INFINITY ? m + logf(z) : -INFINITY;
            }
        }
        __syncthreads();
    }

    // ---- the root against the prefix + self block (never empty)
    if (tid == 0) {
        const float a_root = nd[0].scale * node_l[0];
        const float mx = fmaxf(a_root, l_other);
        const float ltot = mx + logf(expf(a_root - mx) + expf(l_other - mx));
        s_ltot = ltot;
        node_w[0] = a_root > -INFINITY ? a_root - ltot : -INFINITY;
    }
    __syncthreads();
    const float ltot = s_ltot;

    // ---- top-down: log-weights of nodes, and of splits in place of their LogSumExps
    for (int lv = 0; lv < a.n_levels; ++lv) {
        const int n0 = kernarg<TreeMergeArgs>()->level_start[lv], n1 = kernarg<TreeMergeArgs>()->level_start[lv + 1];
        const bool per_thread = n1 - n0 >= kWave;
        for (int n = n0 + (per_thread ? tid : wave); n < n1; n += per_thread ? NT : kMergeWaves) {
            const int cn = child_count(t, n_splits, n);
            const float w_n = node_w[n], l_n = node_l[n];
            const bool leaf = nd[n].leaf_children != 0;
            for (int i = per_thread ? 0 : lane; i < cn; i += per_thread ? 1 : kWave) {
                const float v = child_value(t, n, i);
                const float w = (w_n > -INFINITY && v > -INFINITY) ? w_n + v - l_n : -INFINITY;
                if (leaf) split_v[first_split[n] + i] = w; else node_w[nd[n].first + i] = w;
            }
        }
        __syncthreads();
    }

    // ---- weighted sum of the split results; index n_used stands for the prefix + self block
    float acc[kMaxDimRegs];
#pragma unroll
    for (int r = 0; r < kMaxDimRegs; ++r) acc[r] = 0.f;
    for (int s0 = 0; s0 <= n_used; s0 += kWave) {
        const int s = s0 + lane;
        float w_mine = 0.f;
        if (s < n_used) w_mine = expf(split_v[s]);                 // exp(-inf) = 0
        else if (s == n_used) w_mine = expf(l_other - ltot);
        const int cnt = min(kWave, n_used + 1 - s0);
        // four rows in flight per wavefront; a row of weight zero (an empty split, a slot past the
        // end) is replaced by the prefix+self row, which always holds finite values
        constexpr int UN = 4;
        for (int i = wave; i < cnt; i += UN * kMergeWaves) {
            float w[UN];
            const float* o[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int ii = i + u * kMergeWaves;
                w[u] = ii < cnt ? __shfl(w_mine, min(ii, kWave - 1)) : 0.f;
                const int sp = (w[u] != 0.f && s0 + ii < n_used) ? s0 + ii : a.max_splits;
                o[u] = a.part_o + ((long)sp * U + unit) * d;
            }
            float v[UN][kMaxDimRegs];
#pragma unroll
            for (int u = 0; u < UN; ++u)
#pragma unroll
                for (int r = 0; r < kMaxDimRegs; ++r) {
                    const int c = lane + kWave * r;
                    v[u][r] = c < d ? o[u][c] : 0.f;
                }
#pragma unroll
            for (int u = 0; u < UN; ++u)
#pragma unroll
                for (int r = 0; r < kMaxDimRegs; ++r) acc[r] = fmaf(w[u], v[u][r], acc[r]);
        }
    }
#pragma unroll
    for (int r = 0; r < kMaxDimRegs; ++r) part[wave][lane + kWave * r] = acc[r];
    __syncthreads();
    if (wave != 0) return;
    T* out = (T*)a.out + (long)unit * d;
#pragma unroll
    for (int r = 0; r < kMaxDimRegs; ++r) {
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < kMergeWaves; ++w) v += part[w][lane + kWave * r];
        const int c = lane + kWave * r;
        if (c < d) out[c] = (T)v;
    }
    if (a.lse_out && lane == 0) {
        const int h = unit % a.n_q_heads, row = unit / a.n_q_heads;
        a.lse_out[(long)h * a.q_len + row] = ltot;
    }
}

// The same tree merge for MANY units of a small tree (a query prefill: 8192 units): one WAVEFRONT per
// unit, four units per workgroup.  The tree's bookkeeping (nodes, first split and split count of every
// node) is read once per workgroup and shared; every wavefront has its own node and split values in
// LDS and walks the levels with no workgroup barrier (the LDS operations of one wavefront complete
// in order; the fences below only keep the compiler from moving them).  The workgroup-per-unit
// kernel above spends 19-38 us on 8192 units of a 1- or 9-node tree, most of it barriers and launches.
constexpr int kTreeUnitsPerBlock = 4;
// a level of at least this many nodes gives every lane a node (children read serially); a narrower one
// takes its nodes one after the other with the children across the lanes (the root and its 64 contexts)
constexpr int kLanePerNodeMin = 4;
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}
__host__ __device__ inline size_t tree_wave_lds_bytes(int n_nodes, int max_splits) {
    return (size_t)n_nodes * (sizeof(ape_tree_node) + 2 * sizeof(int)) +
           (size_t)kTreeUnitsPerBlock * ((size_t)n_nodes * 2 * sizeof(float) + (size_t)max_splits * sizeof(float));
}

// D128: head_dim is 128 and a lane owns dims 2 lane, 2 lane + 1 (one 8-byte load per row); otherwise dims
// lane + 64 r as in the kernel above.
template <typename T, bool D128>
__global__ __launch_bounds__(kWave * kTreeUnitsPerBlock) void tree_merge_wave_kernel(const TreeMergeArgs a) {
    extern __shared__ __attribute__((aligned(16))) char tree_lds[];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    constexpr int NT = kWave * kTreeUnitsPerBlock;
    const int d = a.head_dim, U = a.units_total, n_nodes = a.n_nodes;
    const bool valid = (int)blockIdx.x * kTreeUnitsPerBlock + wave < U;
    const int unit = valid ? (int)blockIdx.x * kTreeUnitsPerBlock + wave : U - 1;   // (a spare wavefront recomputes the last unit and stores nothing)
    const TreePlanLayout lay{a.n_nodes, a.max_splits};
    const int n_used = a.plan[0];

    ape_tree_node* nd = (ape_tree_node*)tree_lds;                  // [n_nodes], shared
    int* first_split = (int*)(nd + n_nodes);                       // [n_nodes], shared
    int* n_splits = first_split + n_nodes;                         // [n_nodes], shared
    float* mine = (float*)(n_splits + n_nodes) + (size_t)wave * (2 * n_nodes + a.max_splits);
    float* node_l = mine;                                          // [n_nodes] LogSumExp of the children's values
    float* node_w = node_l + n_nodes;                              // [n_nodes] log-weight in the result
    float* split_v = node_w + n_nodes;                             // [max_splits] LogSumExp, later log-weight

    for (int n = tid; n < n_nodes; n += NT) {
        nd[n] = a.nodes[n];
        first_split[n] = a.plan[lay.first_split_at() + n];
        n_splits[n] = a.plan[lay.n_splits_at() + n];
    }
    for (int s = lane; s < n_used; s += kWave) split_v[s] = a.part_lse[(long)s * U + unit];
    const float l_other = a.part_lse[(long)a.max_splits * U + unit];
    __syncthreads();                                               // the only workgroup barrier: the shared bookkeeping
    const TreeLds t{nd, first_split, node_l, split_v};

    // ---- bottom-up
    for (int lv = a.n_levels - 1; lv >= 0; --lv) {
        const int n0 = kernarg<TreeMergeArgs>()->level_start[lv], n1 = kernarg<TreeMergeArgs>()->level_start[lv + 1];
        if (n1 - n0 >= kLanePerNodeMin) {
            for (int n = n0 + lane; n < n1; n += kWave) {
                const int cn = child_count(t, n_splits, n);
                float m = -INFINITY;
                for (int i = 0; i < cn; ++i) m = fmaxf(m, child_value(t, n, i));
                float z = 0.f;
                if (m > -INFINITY)
                    for (int i = 0; i < cn; ++i) z += expf(child_value(t, n, i) - m);
                node_l[n] = m > -INFINITY ? m + logf(z) : -INFINITY;
            }
        } else {
            for (int n = n0; n < n1; ++n) {
                const int cn = child_count(t, n_splits, n);
                float m = -INFINITY;
                for (int i = lane; i < cn; i += kWave) m = fmaxf(m, child_value(t, n, i));
                m = wave_max(m);
                float z = 0.f;
                if (m > -INFINITY)
                    for (int i = lane; i < cn; i += kWave) z += expf(child_value(t, n, i) - m);
                z = wave_sum(z);
                if (lane == 0) node_l[n] = m > -INFINITY ? m + logf(z) : -INFINITY;
            }
        }
        wave_lds_sync();
    }

    // ---- the root against the prefix + self block (never empty); every lane computes the same
    const float a_root = nd[0].scale * node_l[0];
    const float mx = fmaxf(a_root, l_other);
    const float ltot = mx + logf(expf(a_root - mx) + expf(l_other - mx));
    if (lane == 0) node_w[0] = a_root > -INFINITY ? a_root - ltot : -INFINITY;
    wave_lds_sync();

    // ---- top-down: log-weights of nodes, and of splits in place of their LogSumExps
    for (int lv = 0; lv < a.n_levels; ++lv) {
        const int n0 = kernarg<TreeMergeArgs>()->level_start[lv], n1 = kernarg<TreeMergeArgs>()->level_start[lv + 1];
        const bool per_thread = n1 - n0 >= kLanePerNodeMin;
        for (int n = n0 + (per_thread ? lane : 0); n < n1; n += per_thread ? kWave : 1) {
            const int cn = child_count(t, n_splits, n);
            const float w_n = node_w[n], l_n = node_l[n];
            const bool leaf = nd[n].leaf_children != 0;
            for (int i = per_thread ? 0 : lane; i < cn; i += per_thread ? 1 : kWave) {
                const float v = child_value(t, n, i);
                const float w = (w_n > -INFINITY && v > -INFINITY) ? w_n + v - l_n : -INFINITY;
                if (leaf) split_v[first_split[n] + i] = w; else node_w[nd[n].first + i] = w;
            }
        }
        wave_lds_sync();
    }

    // ---- weighted sum of the split results; index n_used stands for the prefix + self block
    constexpr int DR = D128 ? 2 : kMaxDimRegs;
    float acc[DR];
#pragma unroll
    for (int r = 0; r < DR; ++r) acc[r] = 0.f;
    for (int s0 = 0; s0 <= n_used; s0 += kWave) {
        const int s = s0 + lane;
        float w_mine = 0.f;
        if (s < n_used) w_mine = expf(split_v[s]);                 // exp(-inf) = 0
        else if (s == n_used) w_mine = expf(l_other - ltot);
        const int cnt = min(kWave, n_used + 1 - s0);
        // eight rows in flight; a row of weight zero (an empty split, a slot past the end) is
        // replaced by the prefix+self row, which always holds finite values
        constexpr int UN = 8;
        for (int i = 0; i < cnt; i += UN) {
            float w[UN];
            const float* o[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int ii = i + u;
                w[u] = ii < cnt ? __shfl(w_mine, min(ii, kWave - 1)) : 0.f;
                const int sp = (w[u] != 0.f && s0 + ii < n_used) ? s0 + ii : a.max_splits;
                o[u] = a.part_o + ((long)sp * U + unit) * d;
            }
            float v[UN][DR];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                if constexpr (D128) {
                    const float2 x = *(const float2*)(o[u] + 2 * lane);
                    v[u][0] = x.x; v[u][1] = x.y;
                } else {
#pragma unroll
                    for (int r = 0; r < DR; ++r) {
                        const int c = lane + kWave * r;
                        v[u][r] = c < d ? o[u][c] : 0.f;
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < UN; ++u)
#pragma unroll
                for (int r = 0; r < DR; ++r) acc[r] = fmaf(w[u], v[u][r], acc[r]);
        }
    }
    if (!valid) return;
    T* out = (T*)a.out + (long)unit * d;
    if constexpr (D128) {
        if constexpr (sizeof(T) == 4) {
            *(float2*)(out + 2 * lane) = make_float2(acc[0], acc[1]);
        } else {
            const T o2[2] = {(T)acc[0], (T)acc[1]};
            *(uint32_t*)(out + 2 * lane) = *(const uint32_t*)o2;
        }
    } else {
#pragma unroll
        for (int r = 0; r < DR; ++r) {
            const int c = lane + kWave * r;
            if (c < d) out[c] = (T)acc[r];
        }
    }
    if (a.lse_out && lane == 0) {
        const int h = unit % a.n_q_heads, row = unit / a.n_q_heads;
        a.lse_out[(long)h * a.q_len + row] = ltot;
    }
}

}  // namespace

hipError_t launch_generic_query(const QueryArgs& a, int dtype, hipStream_t s) {
    dim3 grid((unsigned)(a.n_req * a.q_len * a.n_q_heads), (unsigned)(a.n_ctx_splits + 1));
    if (dtype == APE_F32) generic_query_kernel<float><<<grid, kWave, 0, s>>>(a);
    else generic_query_kernel<__bf16><<<grid, kWave, 0, s>>>(a);
    return hipGetLastError();
}

hipError_t launch_generic_encode(const EncodeArgs& a, int dtype, hipStream_t s) {
    if (a.total_rows == 0) return hipSuccess;
    dim3 grid((unsigned)((long)a.total_rows * a.n_q_heads));
    if (dtype == APE_F32) generic_encode_kernel<float><<<grid, kWave, 0, s>>>(a);
    else generic_encode_kernel<__bf16><<<grid, kWave, 0, s>>>(a);
    return hipGetLastError();
}

hipError_t launch_merge(const MergeArgs& a, hipStream_t s) {
    dim3 grid((unsigned)(a.n_req * a.q_len * a.n_q_heads));
    const bool few = a.n_ctx_splits >= 32 && (long)grid.x * a.n_splits_total <= 4096;
    if (!few && a.head_dim == 128 && grid.x >= 256 && a.n_splits_total <= 65) {
        const unsigned blocks = (grid.x + kMergeUnitsPerBlock - 1) / kMergeUnitsPerBlock;
        if (a.dtype == APE_F32) merge_units_kernel<float><<<blocks, 256, 0, s>>>(a);
        else merge_units_kernel<__bf16><<<blocks, 256, 0, s>>>(a);
        return hipGetLastError();
    }
    if (a.dtype == APE_F32) {
        if (few) merge_kernel<float, kMergeWavesFew><<<grid, kWave * kMergeWavesFew, 0, s>>>(a);
        else merge_kernel<float, kMergeWaves><<<grid, kWave * kMergeWaves, 0, s>>>(a);
    } else {
        if (few) merge_kernel<__bf16, kMergeWavesFew><<<grid, kWave * kMergeWavesFew, 0, s>>>(a);
        else merge_kernel<__bf16, kMergeWaves><<<grid, kWave * kMergeWaves, 0, s>>>(a);
    }
    return hipGetLastError();
}

hipError_t launch_tree_plan(const TreePlanArgs& a, hipStream_t s) {
    tree_plan_kernel<<<1, kPlanThreads, 0, s>>>(a);
    return hipGetLastError();
}

hipError_t launch_tree_merge(const TreeMergeArgs& a, hipStream_t s) {
    // many units of a small tree: a wavefront per unit
    const size_t wave_lds = tree_wave_lds_bytes(a.n_nodes, a.max_splits);
    if (a.units_total >= 256 && wave_lds <= 32 * 1024) {
        dim3 wgrid((unsigned)((a.units_total + kTreeUnitsPerBlock - 1) / kTreeUnitsPerBlock));
        const unsigned nt = kWave * kTreeUnitsPerBlock;
        if (a.head_dim == 128) {
            if (a.dtype == APE_F32) tree_merge_wave_kernel<float, true><<<wgrid, nt, wave_lds, s>>>(a);
            else tree_merge_wave_kernel<__bf16, true><<<wgrid, nt, wave_lds, s>>>(a);
        } else {
            if (a.dtype == APE_F32) tree_merge_wave_kernel<float, false><<<wgrid, nt, wave_lds, s>>>(a);
            else tree_merge_wave_kernel<__bf16, false><<<wgrid, nt, wave_lds, s>>>(a);
        }
        return hipGetLastError();
    }
    dim3 grid((unsigned)a.units_total);
    const size_t lds = (size_t)a.n_nodes * (sizeof(ape_tree_node) + 4 * sizeof(float)) + (size_t)a.max_splits * sizeof(float);
    hipError_t e;
    if (a.dtype == APE_F32) {
        e = hipFuncSetAttribute((const void*)tree_merge_kernel<float>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        tree_merge_kernel<float><<<grid, kWave * kMergeWaves, lds, s>>>(a);
    } else {
        e = hipFuncSetAttribute((const void*)tree_merge_kernel<__bf16>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        tree_merge_kernel<__bf16><<<grid, kWave * kMergeWaves, lds, s>>>(a);
    }
    return hipGetLastError();
}

}  // namespace ape
