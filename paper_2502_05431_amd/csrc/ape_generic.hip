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
        long t0 = (long)split * a.ctx_split_len;
        const long t1 = min((long)kv.total_ctx, t0 + a.ctx_split_len);
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

// One group of splits [s0, s1): this wavefront's share of sum_s w_s o_s into acc (lane owns dims
// lane + 64 r), with w_s = exp(lse_s - max); returns the group's max and sum of weights.
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
            for (int i = wave; i < cnt; i += kMergeWaves) {
                const float w = __shfl(w_mine, i);
                const float* o = a.part_o + ((long)(c0 + i) * a.units_total + gunit) * d;
#pragma unroll
                for (int r = 0; r < kMaxDimRegs; ++r) {
                    const int c = lane + kWave * r;
                    if (c < d) acc[r] = fmaf(w, o[c], acc[r]);
                }
            }
        }
        z = wave_sum(z);
    }
    m_out = m; z_out = z;
}

template <typename T>
__global__ __launch_bounds__(kWave * kMergeWaves) void merge_kernel(const MergeArgs a) {
    __shared__ float part[2][kMergeWaves][kWave * kMaxDimRegs];
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
    merge_group(a, gunit, 0, a.n_ctx_splits, wave, lane, acc_c, mc, zc);                  // context group
    merge_group(a, gunit, a.n_ctx_splits, a.n_splits_total, wave, lane, acc_o, mo, zo);   // prefix + self: never empty
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
        for (int w = 0; w < kMergeWaves; ++w) { acc_c[r] += part[0][w][lane + kWave * r]; acc_o[r] += part[1][w][lane + kWave * r]; }
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
        if (a.lse_head_major) {
            const int h = unit % hq, row = (unit / hq) % a.q_len;
            a.lse_out[(long)h * a.q_len + row] = lse;
        } else {
            a.lse_out[gunit] = lse;
        }
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
    if (a.dtype == APE_F32) merge_kernel<float><<<grid, kWave * kMergeWaves, 0, s>>>(a);
    else merge_kernel<__bf16><<<grid, kWave * kMergeWaves, 0, s>>>(a);
    return hipGetLastError();
}

}  // namespace ape
