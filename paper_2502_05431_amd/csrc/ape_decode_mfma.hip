// Bandwidth-bound decode attention for gfx950 (bf16, head_dim 128, one query row per request).
//
// Math (arXiv 2502.05431): Section 4.4 refined attention for a single query row, evaluated as
// blocks (Appendix C.1).  A workgroup owns one (request, KV head, split of the keys); its result
// is a softmax-weighted value vector plus LogSumExp; the merge kernel pools the context splits,
// applies S to the pooled context LogSumExp and merges with prefix + self (Appendix C.3/C.4).
//
// The kernel streams K and V once from HBM; the G query heads of the KV head ride on the same
// loads.  The dot products run on the matrix cores (MFMA 16x16x32 bf16) so that the vector ALUs
// only carry the softmax:
//   S^T[token, head] = K[16 tokens x 128] Q^T[128 x 16 heads]   (heads >= G are zero columns)
//   O[head, dim]    += P[head, 32 tokens] V[32 tokens, 16 dims]
// The accumulator layout of S^T (lane = head, registers = tokens) is exactly the A-operand
// layout of P, with the tokens of a 32-token tile permuted; V is gathered straight from global
// memory in that same permuted order (4-byte loads of a dim pair from 8 token rows, then a byte
// permute splits even and odd dims), so neither P nor V is transposed through LDS.
// Each wavefront streams its own tokens with one tile (16 KB) of loads in flight behind the
// tile being computed; the four wavefronts of a workgroup combine their states in LDS at the end.
#include "ape_internal.h"

#define APE_STREAM_FN __device__ __forceinline__
#define ape_stream_load_i32 ::ape::scalar_load_i32
#define ape_stream_load_ptr ::ape::scalar_load_ptr
#define ape_stream_find_chunk ::ape::find_chunk
#include "ape_decode_stream.h"

#include <math.h>

namespace ape {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int D = 128;
constexpr int ROWB = D * 2;
constexpr int NT = 256;
constexpr int NW = NT / 64;
static_assert(NW == kDecodeWaves, "the stream bookkeeping deals a split to four wavefronts");
constexpr int BT = kDecodeTile;                // tokens per wavefront tile
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

// Loads of one tile (n_valid in 1..32 tokens starting at kb/vb for this KV head).  Rows past
// n_valid are clamped to the last valid row: finite data whose probabilities are zero.
//   k[x*4 + s]: token 16x + (lane & 15), dims 32s + 8*(lane >> 4) .. +7
//   v[pb*8 + e]: k-slot e of this lane's token group, dims 32pb + 2*(lane & 15) + {0,1}
__device__ __forceinline__ void load_k(const char* kb, int n_valid, long stride_b, u32x4 (&k)[8]) {
    const int lane = threadIdx.x & 63;
    const int l16 = lane & 15, kg = lane >> 4;
#pragma unroll
    for (int x = 0; x < 2; ++x) {
        const int row = min(16 * x + l16, n_valid - 1);
        const char* p = kb + (long)row * stride_b + kg * 16;
#pragma unroll
        for (int s = 0; s < 4; ++s) k[x * 4 + s] = *(const u32x4*)(p + s * 64);
    }
}
__device__ __forceinline__ void load_v(const char* vb, int n_valid, long stride_b, uint32_t (&v)[32]) {
    const int lane = threadIdx.x & 63;
    const int l16 = lane & 15, kg = lane >> 4;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int tok = min((e < 4 ? 4 * kg + e : 16 + 4 * kg + (e - 4)), n_valid - 1);
        const char* p = vb + (long)tok * stride_b + l16 * 4;
#pragma unroll
        for (int pb = 0; pb < 4; ++pb) v[pb * 8 + e] = *(const uint32_t*)(p + pb * 64);
    }
}

struct WaveState {
    float m;             // running max (log2 units) of head lane & 15
    float l;             // this lane's share of the running sum
    f32x4 o[8];          // [pb*2 + parity]: head 4*(lane >> 4) + r, dim 32pb + 2*(lane & 15) + parity
};

// S^T = K Q^T for one tile, then the online softmax; returns P (A operand of the PV product).
__device__ __forceinline__ bf16x8 scores_softmax(const u32x4 (&k)[8], int n_valid, const bf16x8 (&qf)[4], float sc2, WaveState& st) {
    const int lane = threadIdx.x & 63;
    const int kg = lane >> 4;
    f32x4 s[2];
#pragma unroll
    for (int x = 0; x < 2; ++x) {
        s[x] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            s[x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, k[x * 4 + ks]), qf[ks], s[x], 0, 0, 0);
    }
    // register r of half x holds token 16x + 4*kg + r for head (lane & 15)
    if (n_valid < BT) {
#pragma unroll
        for (int x = 0; x < 2; ++x)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (16 * x + 4 * kg + r >= n_valid) s[x][r] = -INFINITY;
    }
    float mx = fmaxf(fmaxf(fmaxf(s[0][0], s[0][1]), fmaxf(s[0][2], s[0][3])),
                     fmaxf(fmaxf(s[1][0], s[1][1]), fmaxf(s[1][2], s[1][3])));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(st.m, mx * sc2);              // finite: token 0 of the tile is valid
    const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);
    bf16x8 p;
    float psum = 0.f;
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float pv = __builtin_amdgcn_exp2f(fmaf(s[x][r], sc2, -m_new));
            psum += pv;
            p[4 * x + r] = (__bf16)pv;
        }
    st.l = st.l * alpha + psum;
    st.m = m_new;
    // rescale O: its rows are heads 4*kg + r, whose alpha lives in lane (4*kg + r)
    if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float ar = __shfl(alpha, 4 * kg + r);
#pragma unroll
            for (int i = 0; i < 8; ++i) st.o[i][r] *= ar;
        }
    }
    return p;
}

// O += P V, even and odd dims of each pair block
__device__ __forceinline__ void accumulate_pv(const uint32_t (&v)[32], bf16x8 p, WaveState& st) {
#pragma unroll
    for (int pb = 0; pb < 4; ++pb) {
        u32x4 ev, od;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t w0 = v[pb * 8 + 2 * u], w1 = v[pb * 8 + 2 * u + 1];
            ev[u] = __builtin_amdgcn_perm(w1, w0, 0x05040100u);     // lo16(w0) | lo16(w1) << 16
            od[u] = __builtin_amdgcn_perm(w1, w0, 0x07060302u);     // hi16(w0) | hi16(w1) << 16
        }
        st.o[pb * 2 + 0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(p, __builtin_bit_cast(bf16x8, ev), st.o[pb * 2 + 0], 0, 0, 0);
        st.o[pb * 2 + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(p, __builtin_bit_cast(bf16x8, od), st.o[pb * 2 + 1], 0, 0, 0);
    }
}

// Software pipeline of one wavefront: the K registers are refilled for the next tile as soon as
// the score MFMAs have consumed them, the V registers as soon as the PV MFMAs have.
__device__ __forceinline__ void run_stream(DecodeStream& sm, long stride_b, const bf16x8 (&qf)[4], float sc2, WaveState& st) {
    const char *kb, *vb, *kn, *vn;
    int nv, nn;
    if (!sm.next(kb, vb, nv)) return;
    u32x4 k[8];
    uint32_t v[32];
    load_k(kb, nv, stride_b, k);
    load_v(vb, nv, stride_b, v);
    bool more = true;
    while (more) {
        more = sm.next(kn, vn, nn);
        const bf16x8 p = scores_softmax(k, nv, qf, sc2, st);
        if (more) load_k(kn, nn, stride_b, k);
        accumulate_pv(v, p, st);
        if (more) load_v(vn, nn, stride_b, v);
        nv = nn;
    }
}

// grid: x = split (context splits, then prefix + self), y = KV head, z = request in this launch
template <int G>
__global__ __launch_bounds__(NT, 2) void decode_kernel(const QueryArgs a, const bool head_fastest) {
    __shared__ float sm_m[NW][16];
    __shared__ float sm_l[NW][16];
    __shared__ float sm_o[NW][G][D];
    // the wavefront index is made provably uniform: everything the block walker derives from it
    // (token ranges, chunk indices, table addresses) then lives in scalar registers and its
    // branches are scalar branches -- a scalar table load must never sit in divergent control
    // flow, where it would run with EXEC = 0 and a stale address
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l16 = lane & 15, kg = lane >> 4;
    // Two dispatch orders (x is the fastest index).  When the whole grid is resident at once, KV head
    // fastest: the heads of one (request, split) start together and walk the same [token, head, d]
    // rows in step, so a token's 2 KB row comes from one open DRAM page (measured: 128K context,
    // batch 1, 114 -> 108 us).  With several rounds of workgroups the heads drift apart and that
    // order only concentrates every XCD on one head's addresses (batch 32: 385 -> 410 us), so the
    // split index stays fastest there.
    int hk, split;
    if (head_fastest) { hk = blockIdx.x; split = blockIdx.y; }
    else { split = blockIdx.x; hk = blockIdx.y; }
    const int rq = blockIdx.z;
    // the request descriptor is read straight from the kernel-argument segment (scalar loads);
    // indexing the by-value argument with a run-time index would copy all of it to scratch
    const KvView kv = load_view<QueryArgs>(rq);
    const int hq = a.n_q_heads;
    const long stride_b = (long)a.n_kv_heads * ROWB, head_b = (long)hk * ROWB;

    // Q^T as B operand: column = head l16 (zero beyond G), dims 32*ks + 8*kg .. +7
    bf16x8 qf[4];
    {
        const char* qp = (const char*)a.q + ((long)rq * hq + hk * G + l16) * ROWB + kg * 16;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            u32x4 w = {0, 0, 0, 0};
            if (l16 < G) w = *(const u32x4*)(qp + ks * 64);
            qf[ks] = __builtin_bit_cast(bf16x8, w);
        }
    }
    WaveState st;
    st.m = -INFINITY; st.l = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) st.o[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
    const float inv_sqrt_d = 0.08838834764831845f;

    DecodeStream sm;
    if (split < a.n_ctx_splits) {
        long t0, t1, lo, hi;
        ctx_split_range(a, kv, split, t0, t1);
        decode_wave_share(t0, t1, wave, lo, hi);
        sm.init_ctx(kv, lo, hi, stride_b, head_b);
        run_stream(sm, stride_b, qf, inv_sqrt_d / kv.temperature * LOG2E, st);
    } else {
        // prefix + self (one query row sees all self_len tokens)
        int pb, pe, sb, se;
        decode_plain_shares(kv.prefix_len, kv.self_len, wave, pb, pe, sb, se);
        sm.init_plain((const char*)kv.k_prefix + (long)pb * stride_b + head_b, (const char*)kv.v_prefix + (long)pb * stride_b + head_b, pe - pb,
                      (const char*)kv.k_self + (long)sb * stride_b + head_b, (const char*)kv.v_self + (long)sb * stride_b + head_b, se - sb,
                      stride_b);
        run_stream(sm, stride_b, qf, inv_sqrt_d * LOG2E, st);
    }

    // ---- combine the four wavefronts (Appendix C.1 merge of their blocks)
    float lt = st.l + __shfl_xor(st.l, 16);
    lt += __shfl_xor(lt, 32);
    if (kg == 0) { sm_m[wave][l16] = st.m; sm_l[wave][l16] = lt; }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int head = 4 * kg + r;
        if (head < G) {
#pragma unroll
            for (int pb = 0; pb < 4; ++pb) {
                sm_o[wave][head][32 * pb + 2 * l16 + 0] = st.o[pb * 2 + 0][r];
                sm_o[wave][head][32 * pb + 2 * l16 + 1] = st.o[pb * 2 + 1][r];
            }
        }
    }
    __syncthreads();
    const long unit0 = ((long)a.req_base + rq) * hq + hk * G;          // q_len == 1
    for (int idx = threadIdx.x; idx < G * D; idx += NT) {
        const int g = idx / D, c = idx % D;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < NW; ++w) M = fmaxf(M, sm_m[w][g]);
        float L = 0.f, O = 0.f;
        if (M > -INFINITY) {
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const float f = __builtin_amdgcn_exp2f(sm_m[w][g] - M);   // 0 for an idle wavefront
                L += sm_l[w][g] * f;
                O += sm_o[w][g][c] * f;
            }
        }
        const long slot = (long)split * a.units_total + unit0 + g;
        a.part_o[slot * D + c] = L > 0.f ? O / L : 0.f;
        if (c == 0) a.part_lse[slot] = L > 0.f ? (M + __builtin_amdgcn_logf(L)) * LN2 : -INFINITY;
    }
}

}  // namespace

hipError_t launch_decode_mfma(const QueryArgs& a, hipStream_t s) {
    const int group = a.n_q_heads / a.n_kv_heads;
    // workgroups that fit on the chip at once: two per CU (launch bounds), 256 CUs
    const long total = (long)a.n_kv_heads * (a.n_ctx_splits + 1) * a.n_req;
    const bool hf = total <= 2 * 256 + 64;
    const dim3 grid = hf ? dim3((unsigned)a.n_kv_heads, (unsigned)(a.n_ctx_splits + 1), (unsigned)a.n_req)
                         : dim3((unsigned)(a.n_ctx_splits + 1), (unsigned)a.n_kv_heads, (unsigned)a.n_req);
    switch (group) {
        case 1: decode_kernel<1><<<grid, NT, 0, s>>>(a, hf); break;
        case 2: decode_kernel<2><<<grid, NT, 0, s>>>(a, hf); break;
        case 4: decode_kernel<4><<<grid, NT, 0, s>>>(a, hf); break;
        default: decode_kernel<8><<<grid, NT, 0, s>>>(a, hf); break;
    }
    return hipGetLastError();
}

}  // namespace ape
