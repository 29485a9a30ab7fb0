// Matrix-core flash attention for gfx950 (bf16, head_dim 128): query prefill over the cached
// contexts (split over the keys) and the block-diagonal causal encoding of the contexts.
//
// Math (arXiv 2502.05431): Section 2.3 softmax attention evaluated block by block as in
// Appendix C.1 (each block: softmax-weighted values + LogSumExp); context blocks use scores
// q.k/(T sqrt d) (Section 4.4); the scaling factor S is applied later, by the merge kernel, to
// the pooled context LogSumExp (Appendix C.3/C.4).
//
// Tiling (wave64, MFMA 32x32x16 bf16):
//   - a workgroup = 4 wavefronts; a wavefront owns RB blocks of 32 query rows, where a "row" is
//     a (query token, head of the GQA group) pair, so the G query heads that share a KV head
//     also share every K/V tile staged in LDS;
//   - keys/values are streamed in tiles of 64 tokens through a double-buffered LDS stage
//     (16-byte coalesced global loads -> registers -> XOR-swizzled LDS rows of 256 bytes);
//   - scores are computed TRANSPOSED, S^T = K Q^T: the accumulator layout then puts one query
//     row in one lane (and its partner lane +32), so the softmax row reductions are in-lane,
//     and the bf16 probabilities are already laid out as the B operand of O^T += V^T P^T;
//   - V^T fragments come from LDS through the transposing read ds_read_b64_tr_b16.
#include "ape_internal.h"

#include <math.h>

namespace ape {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int D = 128;                       // head_dim
constexpr int BN = 64;                       // KV tokens per LDS tile
constexpr int TB = BN / 32;                  // 32-token blocks per tile
constexpr int NT = 256;                      // threads per workgroup
constexpr int NW = NT / 64;                  // wavefronts
constexpr int ROWB = D * 2;                  // bytes of one head's K or V row
constexpr int TILEB = BN * ROWB;             // 16 KB
constexpr int STAGEB = 2 * TILEB;            // K tile + V tile
constexpr int LDSB = 2 * STAGEB;             // double buffer: 64 KB
constexpr int LD_PER_THREAD = BN * 16 / NT;  // 16-byte pieces per thread per tile (4)
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

typedef __attribute__((address_space(3))) char lds_char;

// One KV tile: n_valid (1..BN) consecutive tokens of one segment.
struct Tile {
    const char* k;        // row 0 of the tile for this KV head
    const char* v;
    int n_valid;
    int j0;               // index of row 0 inside the causal segment, or -1 (no causal mask)
};

// Walks the pooled contexts [t0, t1) through the chunk table; tiles stop at chunk ends.
struct CtxWalk {
    const KvView* kv;
    long t, t1, c0, c1;
    int c;
    long stride_b, head_b;
    __device__ void init(const KvView* kv_, long t0_, long t1_, long stride_b_, long head_b_) {
        kv = kv_; t = t0_; t1 = t1_; stride_b = stride_b_; head_b = head_b_;
        c = 0; c0 = 0; c1 = 0;
        if (t < t1) {
            int lo = 0, hi = kv->n_chunks - 1;
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (kv->cu[mid] <= t) lo = mid; else hi = mid - 1;
            }
            c = lo; c0 = kv->cu[c]; c1 = kv->cu[c + 1];
        }
    }
    __device__ bool next(Tile& tile) {
        if (t >= t1) return false;
        while (t >= c1) {                                          // next non-empty chunk
            if (c + 1 >= kv->n_chunks) { t = t1; return false; }   // table shorter than total_ctx: stop, stay in bounds
            ++c; c0 = c1; c1 = kv->cu[c + 1];
        }
        const long e = c1 < t1 ? c1 : t1;
        const int n = (int)(e - t < BN ? e - t : BN);
        tile.k = (const char*)kv->k_chunks[c] + (t - c0) * stride_b + head_b;
        tile.v = (const char*)kv->v_chunks[c] + (t - c0) * stride_b + head_b;
        tile.n_valid = n; tile.j0 = -1;
        t += n;
        return true;
    }
};

// Walks a plain segment (the prefix, no mask) and then a causal segment (self KV / own chunk).
struct SeqWalk {
    const char* kp; const char* vp; int np;      // prefix rows
    const char* kc; const char* vc; int nc;      // causal rows visible to this workgroup
    int j; int phase;
    long stride_b;
    __device__ void init(const char* kp_, const char* vp_, int np_, const char* kc_, const char* vc_, int nc_, long stride_b_) {
        kp = kp_; vp = vp_; np = np_; kc = kc_; vc = vc_; nc = nc_; stride_b = stride_b_;
        j = 0; phase = np > 0 ? 0 : 1;
    }
    __device__ bool next(Tile& tile) {
        if (phase == 0) {
            const int n = np - j < BN ? np - j : BN;
            tile.k = kp + (long)j * stride_b; tile.v = vp + (long)j * stride_b; tile.n_valid = n; tile.j0 = -1;
            j += n;
            if (j >= np) { phase = 1; j = 0; }
            return true;
        }
        if (j >= nc) return false;
        const int n = nc - j < BN ? nc - j : BN;
        tile.k = kc + (long)j * stride_b; tile.v = vc + (long)j * stride_b; tile.n_valid = n; tile.j0 = j;
        j += n;
        return true;
    }
};

struct Staged { u32x4 k[LD_PER_THREAD]; u32x4 v[LD_PER_THREAD]; };

// 16-byte pieces: piece id = i*NT + tid -> (row = id / 16, chunk = id % 16); rows past n_valid are zero.
__device__ __forceinline__ void load_tile(const Tile& t, long stride_b, Staged& s) {
    const int tid = threadIdx.x;
#pragma unroll
    for (int i = 0; i < LD_PER_THREAD; ++i) {
        const int id = i * NT + tid;
        const int row = id >> 4, ch = id & 15;
        if (row < t.n_valid) {
            s.k[i] = *(const u32x4*)(t.k + (long)row * stride_b + ch * 16);
            s.v[i] = *(const u32x4*)(t.v + (long)row * stride_b + ch * 16);
        } else {
            s.k[i] = (u32x4){0, 0, 0, 0};
            s.v[i] = (u32x4){0, 0, 0, 0};
        }
    }
}

// K rows: 16-byte chunk index XOR (row & 15): conflict-free 16-byte reads down a column of rows.
// V rows: chunk index XOR 4*(row & 3): the four rows of one transposing read land in distinct
// 64-byte windows.
__device__ __forceinline__ int k_off(int row, int ch) { return row * ROWB + ((ch ^ (row & 15)) << 4); }
__device__ __forceinline__ int v_off(int row, int ch) { return row * ROWB + ((ch ^ ((row & 3) << 2)) << 4); }

__device__ __forceinline__ void store_tile(const Staged& s, char* stage) {
    const int tid = threadIdx.x;
#pragma unroll
    for (int i = 0; i < LD_PER_THREAD; ++i) {
        const int id = i * NT + tid;
        const int row = id >> 4, ch = id & 15;
        *(u32x4*)(stage + k_off(row, ch)) = s.k[i];
        *(u32x4*)(stage + TILEB + v_off(row, ch)) = s.v[i];
    }
}

__device__ __forceinline__ bf16x4 lds_read_tr(const char* p) {
    s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
    return __builtin_bit_cast(bf16x4, r);
}

// Per-wavefront running softmax state of RB blocks of 32 query rows.
template <int RB>
struct WaveState {
    float m[RB];                 // running max, log2 units (score * scale * log2 e)
    float l[RB];                 // this lane's share of the running sum
    f32x16 o[RB][4];             // O^T accumulators: [row block][32-dim block]
};

// One KV tile for one wavefront, 32 tokens at a time: S^T = K Q^T, online softmax, O^T += V^T P^T.
//   qf       Q fragments [RB][8 k-slabs]
//   sc2      score scale * log2(e)
//   lim[rb]  causal limit of this lane's row (largest visible index of the causal segment)
// The running reference maximum m only moves when a row's new maximum exceeds it by more than
// kLazy (log2 units): probabilities then stay below 2^kLazy and the accumulators are rescaled
// only on those rare steps.
constexpr float kLazy = 8.f;

template <int RB>
__device__ __forceinline__ void compute_tile(const char* stage, const bf16x8 (&qf)[RB][8], WaveState<RB>& st,
                                             float sc2, const Tile& t, const int (&lim)[RB], bool need_mask) {
    const int lane = threadIdx.x & 63;
    const int l32 = lane & 31, hi = lane >> 5;
    const int g16 = lane >> 4, s16 = lane & 15;
    const char* vst = stage + TILEB;
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        if (tb * 32 >= t.n_valid) break;                      // nothing but padding in this block
        f32x16 s[RB];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[rb][r] = 0.f;

        // ---- S^T = K Q^T
        const int row = tb * 32 + l32;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 a = *(const bf16x8*)(stage + k_off(row, 2 * ks + hi));
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
                s[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[rb][ks], s[rb], 0, 0, 0);
        }

        // ---- masks (tile tail, causal diagonal); accumulator register r holds token
        //      tb*32 + 8*(r/4) + 4*hi + (r%4) of the tile for query row l32
        if (need_mask) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int tok = tb * 32 + 8 * (r >> 2) + 4 * hi + (r & 3);
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
                    const bool dead = tok >= t.n_valid || (t.j0 >= 0 && t.j0 + tok > lim[rb]);
                    if (dead) s[rb][r] = -INFINITY;
                }
            }
        }

        // ---- online softmax per query row (row = lane & 31, shared with lane ^ 32)
        bf16x8 p[RB][2];
        float alpha[RB];
        bool rescale = false;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            float mx = s[rb][0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[rb][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32)) * sc2;
            const float m_old = st.m[rb];
            const float m_new = mx > m_old + kLazy ? mx : m_old;    // -inf + 8 = -inf: first visible key always moves it
            const float m_use = m_new == -INFINITY ? 0.f : m_new;   // row with nothing visible yet
            alpha[rb] = __builtin_amdgcn_exp2f(m_old - m_use);
            rescale |= m_new != m_old;
            float psum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float pv = __builtin_amdgcn_exp2f(fmaf(s[rb][r], sc2, -m_use));
                psum += pv;
                p[rb][r >> 3][r & 7] = (__bf16)pv;
            }
            st.l[rb] = st.l[rb] * alpha[rb] + psum;
            st.m[rb] = m_new;
        }
        if (__builtin_amdgcn_ballot_w64(rescale) != 0) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) st.o[rb][db][r] *= alpha[rb];
        }

        // ---- O^T += V^T P^T.  k-slot e of lane half `hi` in slab sl is token
        //      tb*32 + 16*sl + (e < 4 ? 4*hi + e : 8 + 4*hi + e - 4): two transposing reads.
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) {
            const int row0 = tb * 32 + 16 * sl + 4 * (g16 >> 1) + (s16 >> 2);
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const int ch = 4 * db + 2 * (g16 & 1) + ((s16 & 3) >> 1);
                const int sub = (s16 & 1) * 8;
                const bf16x4 lo4 = lds_read_tr(vst + v_off(row0, ch) + sub);
                const bf16x4 hi4 = lds_read_tr(vst + v_off(row0 + 8, ch) + sub);
                const bf16x8 a = __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
                    st.o[rb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p[rb][sl], st.o[rb][db], 0, 0, 0);
            }
        }
    }
}

// Streams every tile of `walk` through the double-buffered LDS stage.
//   vis_hi  largest causal index any row of THIS wavefront sees (tiles beyond it are skipped)
//   vis_lo  smallest causal limit among this wavefront's rows (tiles up to it need no causal mask)
template <int RB, typename Walk>
__device__ __forceinline__ void run_tiles(Walk& walk, long stride_b, char* lds, const bf16x8 (&qf)[RB][8],
                                          WaveState<RB>& st, float sc2, const int (&lim)[RB], int vis_lo, int vis_hi) {
    Tile cur, nxt;
    bool have = walk.next(cur);
    Staged sg;
    if (have) load_tile(cur, stride_b, sg);
    int it = 0;
    while (have) {
        char* stage = lds + (it & 1) * STAGEB;
        store_tile(sg, stage);
        __syncthreads();
        const bool have_next = walk.next(nxt);
        if (have_next) load_tile(nxt, stride_b, sg);
        const bool causal = cur.j0 >= 0;
        if (!(causal && cur.j0 > vis_hi)) {
            const bool need_mask = cur.n_valid < BN || (causal && cur.j0 + BN - 1 > vis_lo);
            compute_tile<RB>(stage, qf, st, sc2, cur, lim, need_mask);
        }
        cur = nxt; have = have_next; ++it;
    }
}

template <int RB>
__device__ __forceinline__ void init_state(WaveState<RB>& st) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        st.m[rb] = -INFINITY; st.l[rb] = 0.f;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) st.o[rb][db][r] = 0.f;
    }
}

// XCD-aware work mapping.  Workgroups are dealt round-robin to the 8 XCDs (each with its own
// L2); a "team" = the workgroups that read the same K/V (all query tiles of one KV range).
// Teams are dealt to XCDs so that the members of a team run on one XCD back to back.
__device__ __forceinline__ void team_of_block(int block, int team_size, int& team, int& member) {
    const int xcd = block & 7, slot = block >> 3;
    member = slot % team_size;
    team = (slot / team_size) * 8 + xcd;
}

// ------------------------------------------------------------------------------------------
// Query prefill: grid = 8 * ceil(teams / 8) * n_qtiles, team = (split, KV head).
// Rows: R = qtile*BM + wave*32*RB + rb*32 + (lane & 31); query token = R / G, head = hk*G + R % G.
template <int RB, int G>
__global__ __launch_bounds__(NT) void flash_prefill_kernel(const QueryArgs a, int n_qtiles) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    constexpr int BM = NW * 32 * RB;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, hi = lane >> 5;
    int team, qtile;
    team_of_block(blockIdx.x, n_qtiles, team, qtile);
    const int n_splits_total = a.n_ctx_splits + 1;
    if (team >= n_splits_total * a.n_kv_heads) return;
    const int split = team % n_splits_total, hk = team / n_splits_total;
    const KvView& kv = a.req[0];
    const int hq = a.n_q_heads, q_len = a.q_len;
    const long stride_b = (long)a.n_kv_heads * ROWB, head_b = (long)hk * ROWB;

    // Q fragments (B operand: row = lane & 31, dims 16*ks + 8*hi .. +7)
    bf16x8 qf[RB][8];
    int lim[RB];
    const int causal_off = kv.self_len - q_len;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int R = qtile * BM + wave * 32 * RB + rb * 32 + l32;
        const int tok = R / G, g = R % G;
        const bool valid = tok < q_len;
        lim[rb] = (valid ? tok : q_len - 1) + causal_off;
        const char* qp = (const char*)a.q + ((long)tok * hq + hk * G + g) * ROWB + hi * 16;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            u32x4 w = {0, 0, 0, 0};
            if (valid) w = *(const u32x4*)(qp + ks * 32);
            qf[rb][ks] = __builtin_bit_cast(bf16x8, w);
        }
    }
    const int R_lo = qtile * BM + wave * 32 * RB, R_hi = R_lo + 32 * RB - 1;
    const int tok_lo = min(R_lo / G, q_len - 1), tok_hi = min(R_hi / G, q_len - 1);

    WaveState<RB> st;
    init_state<RB>(st);
    const float inv_sqrt_d = 0.08838834764831845f;      // 1/sqrt(128)
    if (split < a.n_ctx_splits) {
        const long t0 = (long)split * a.ctx_split_len;
        const long t1 = min((long)kv.total_ctx, t0 + a.ctx_split_len);
        CtxWalk walk;
        walk.init(&kv, t0, t1, stride_b, head_b);
        run_tiles<RB>(walk, stride_b, lds, qf, st, inv_sqrt_d / kv.temperature * LOG2E, lim, 0, 0);
    } else {
        // rows of this workgroup see the causal segment up to the last valid row's limit
        const int wg_tok_hi = min((qtile * BM + BM - 1) / G, q_len - 1);
        SeqWalk walk;
        walk.init((const char*)kv.k_prefix + head_b, (const char*)kv.v_prefix + head_b, kv.prefix_len,
                  (const char*)kv.k_self + head_b, (const char*)kv.v_self + head_b, wg_tok_hi + causal_off + 1, stride_b);
        run_tiles<RB>(walk, stride_b, lds, qf, st, inv_sqrt_d * LOG2E, lim, tok_lo + causal_off, tok_hi + causal_off);
    }

    // ---- block result (Appendix C.1): normalised values + natural-log LogSumExp
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int R = qtile * BM + wave * 32 * RB + rb * 32 + l32;
        const int tok = R / G, g = R % G;
        if (tok >= q_len) continue;
        const float lt = st.l[rb] + __shfl_xor(st.l[rb], 32);
        const float inv = lt > 0.f ? 1.f / lt : 0.f;
        const long unit = (long)tok * hq + hk * G + g;
        const long slot = (long)split * a.units_total + unit;
        float* o = a.part_o + slot * D;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                f32x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = st.o[rb][db][4 * q4 + e] * inv;
                *(f32x4*)(o + 32 * db + 8 * q4 + 4 * hi) = w;
            }
        if (hi == 0) a.part_lse[slot] = lt > 0.f ? (st.m[rb] + __builtin_amdgcn_logf(lt)) * LN2 : -INFINITY;
    }
}

// ------------------------------------------------------------------------------------------
// Block-diagonal causal encode: team = (chunk, KV head), members = query tiles of the chunk,
// heaviest (last) tile first.  Writes the final bf16 output.
template <int RB, int G>
__global__ __launch_bounds__(NT) void flash_encode_kernel(const EncodeArgs a, int n_qtiles) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    constexpr int BM = NW * 32 * RB;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, hi = lane >> 5;
    int team, member;
    team_of_block(blockIdx.x, n_qtiles, team, member);
    if (team >= a.n_chunks * a.n_kv_heads) return;
    const int qtile = n_qtiles - 1 - member;
    const int chunk = team / a.n_kv_heads, hk = team % a.n_kv_heads;
    const int c0 = a.cu ? a.cu[chunk] : 0;
    const int len = a.cu ? a.cu[chunk + 1] - c0 : a.total_rows;
    if ((long)qtile * BM >= (long)len * G) return;
    const int hq = a.n_q_heads;
    const long stride_b = (long)a.n_kv_heads * ROWB, head_b = (long)hk * ROWB;

    bf16x8 qf[RB][8];
    int lim[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int R = qtile * BM + wave * 32 * RB + rb * 32 + l32;
        const int tok = R / G, g = R % G;
        const bool valid = tok < len;
        lim[rb] = valid ? tok : len - 1;
        const char* qp = (const char*)a.q + ((long)(c0 + tok) * hq + hk * G + g) * ROWB + hi * 16;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            u32x4 w = {0, 0, 0, 0};
            if (valid) w = *(const u32x4*)(qp + ks * 32);
            qf[rb][ks] = __builtin_bit_cast(bf16x8, w);
        }
    }
    const int R_lo = qtile * BM + wave * 32 * RB, R_hi = R_lo + 32 * RB - 1;
    const int tok_lo = min(R_lo / G, len - 1), tok_hi = min(R_hi / G, len - 1);
    const int wg_tok_hi = min((qtile * BM + BM - 1) / G, len - 1);

    WaveState<RB> st;
    init_state<RB>(st);
    SeqWalk walk;
    walk.init((const char*)a.k_prefix + head_b, (const char*)a.v_prefix + head_b, a.prefix_len,
              (const char*)a.k + (long)c0 * stride_b + head_b, (const char*)a.v + (long)c0 * stride_b + head_b,
              wg_tok_hi + 1, stride_b);
    run_tiles<RB>(walk, stride_b, lds, qf, st, 0.08838834764831845f * LOG2E, lim, tok_lo, tok_hi);

#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int R = qtile * BM + wave * 32 * RB + rb * 32 + l32;
        const int tok = R / G, g = R % G;
        if (tok >= len) continue;
        const float lt = st.l[rb] + __shfl_xor(st.l[rb], 32);
        const float inv = 1.f / lt;                        // a row always sees itself
        const int h = hk * G + g;
        char* o = (char*)a.out + ((long)(c0 + tok) * hq + h) * ROWB;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                bf16x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = (__bf16)(st.o[rb][db][4 * q4 + e] * inv);
                *(bf16x4*)(o + (32 * db + 8 * q4 + 4 * hi) * 2) = w;
            }
        if (a.lse && hi == 0) a.lse[(long)h * a.total_rows + c0 + tok] = (st.m[rb] + __builtin_amdgcn_logf(lt)) * LN2;
    }
}

template <int RB, int G>
hipError_t launch_prefill_t(const QueryArgs& a, unsigned grid, int n_qtiles, hipStream_t s) {
    hipError_t e = hipFuncSetAttribute((const void*)flash_prefill_kernel<RB, G>, hipFuncAttributeMaxDynamicSharedMemorySize, LDSB);
    if (e != hipSuccess) return e;
    flash_prefill_kernel<RB, G><<<grid, NT, LDSB, s>>>(a, n_qtiles);
    return hipGetLastError();
}

template <int RB, int G>
hipError_t launch_encode_t(const EncodeArgs& a, unsigned grid, int n_qtiles, hipStream_t s) {
    hipError_t e = hipFuncSetAttribute((const void*)flash_encode_kernel<RB, G>, hipFuncAttributeMaxDynamicSharedMemorySize, LDSB);
    if (e != hipSuccess) return e;
    flash_encode_kernel<RB, G><<<grid, NT, LDSB, s>>>(a, n_qtiles);
    return hipGetLastError();
}

template <int RB>
hipError_t launch_prefill_g(int group, const QueryArgs& a, unsigned grid, int n_qtiles, hipStream_t s) {
    switch (group) {
        case 1: return launch_prefill_t<RB, 1>(a, grid, n_qtiles, s);
        case 2: return launch_prefill_t<RB, 2>(a, grid, n_qtiles, s);
        case 4: return launch_prefill_t<RB, 4>(a, grid, n_qtiles, s);
        default: return launch_prefill_t<RB, 8>(a, grid, n_qtiles, s);
    }
}

template <int RB>
hipError_t launch_encode_g(int group, const EncodeArgs& a, unsigned grid, int n_qtiles, hipStream_t s) {
    switch (group) {
        case 1: return launch_encode_t<RB, 1>(a, grid, n_qtiles, s);
        case 2: return launch_encode_t<RB, 2>(a, grid, n_qtiles, s);
        case 4: return launch_encode_t<RB, 4>(a, grid, n_qtiles, s);
        default: return launch_encode_t<RB, 8>(a, grid, n_qtiles, s);
    }
}

}  // namespace

int flash_block_rows(int rows_per_kv_head) { return rows_per_kv_head > 128 ? 256 : 128; }

hipError_t launch_flash_prefill(const QueryArgs& a, hipStream_t s) {
    const int group = a.n_q_heads / a.n_kv_heads;
    const int rows = a.q_len * group;
    const int bm = flash_block_rows(rows);
    const int n_qtiles = (rows + bm - 1) / bm;
    const int teams = (a.n_ctx_splits + 1) * a.n_kv_heads;
    const unsigned grid = (unsigned)((teams + 7) / 8 * 8 * n_qtiles);
    return bm == 256 ? launch_prefill_g<2>(group, a, grid, n_qtiles, s) : launch_prefill_g<1>(group, a, grid, n_qtiles, s);
}

hipError_t launch_flash_encode(const EncodeArgs& a, hipStream_t s) {
    if (a.total_rows == 0) return hipSuccess;
    const int group = a.n_q_heads / a.n_kv_heads;
    const int rows = a.max_chunk_len * group;
    const int bm = flash_block_rows(rows);
    const int n_qtiles = (rows + bm - 1) / bm;
    const int teams = a.n_chunks * a.n_kv_heads;
    const unsigned grid = (unsigned)((teams + 7) / 8 * 8 * n_qtiles);
    return bm == 256 ? launch_encode_g<2>(group, a, grid, n_qtiles, s) : launch_encode_g<1>(group, a, grid, n_qtiles, s);
}

}  // namespace ape
