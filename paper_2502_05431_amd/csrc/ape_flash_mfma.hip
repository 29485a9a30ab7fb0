// Matrix-core flash attention for gfx950 (bf16, head_dim 128): query prefill over the cached
// contexts (split over the keys) and the block-diagonal causal encoding of the contexts.
//
// Math (arXiv 2502.05431): Section 2.3 softmax attention evaluated block by block as in
// Appendix C.1 (each block: softmax-weighted values + LogSumExp); context blocks use scores
// q.k/(T sqrt d) (Section 4.4); the scaling factor S is applied later, by the merge kernel, to
// the pooled context LogSumExp (Appendix C.3/C.4).
//
// Tiling (wave64, MFMA 32x32x16 bf16):
//   - a workgroup = 4 wavefronts, one per SIMD; a wavefront owns RB blocks of 32 query rows,
//     where a "row" is a (query token, head of the GQA group) pair, so the G query heads that
//     share a KV head also share every K/V block staged in LDS;
//   - keys/values stream in blocks of 32 tokens through a ring of LDS slots filled by direct
//     global->LDS loads (16 bytes per lane, no staging registers), several blocks ahead of the
//     compute; rows are 256 bytes and XOR-swizzled so that every LDS read is conflict-free;
//   - scores are computed TRANSPOSED, S^T = K Q^T: the accumulator layout then puts one query
//     row in one lane (and its partner lane +32), so the softmax row reductions are in-lane,
//     and the bf16 probabilities are already laid out as the B operand of O^T += V^T P^T;
//   - V^T fragments come from LDS through the transposing read ds_read_b64_tr_b16;
//   - the loop is software-pipelined: while the vector ALUs run the softmax of block j, the
//     matrix cores run O += P V of block j-1 and K Q^T of block j+1.
#include "ape_internal.h"

#include <math.h>

#include <type_traits>

namespace ape {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void glb_void;

constexpr int D = 128;                       // head_dim
constexpr int BLK = 32;                      // KV tokens per block
constexpr int NT = 256;                      // threads per workgroup
constexpr int NW = NT / 64;                  // wavefronts
constexpr int ROWB = D * 2;                  // bytes of one head's K or V row
constexpr int KVB = BLK * ROWB;              // 8 KB: one block of K (or V) rows
constexpr int SLOTB = 2 * KVB;               // K rows then V rows
#ifndef APE_X_RING
#define APE_X_RING 6
#endif
constexpr int RING = APE_X_RING;                      // LDS slots: blocks j, j+1 in use, 4 more in flight
constexpr int LDSB = RING * SLOTB;           // 96 KB
constexpr int LOADS_PER_BLOCK = 4;           // direct-to-LDS load instructions per wavefront per block
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr float kLazy = 40.f;                // the reference maximum moves only when exceeded by 2^kLazy

// One KV block: n_valid (1..32) consecutive tokens of one segment.
struct Block {
    const char* k;        // row 0 of the block for this KV head
    const char* v;
    int n_valid;
    int j0;               // index of row 0 inside the causal segment, or -1 (no causal mask)
};

// Block source of one workgroup.  Two modes share one type (and therefore one instantiation of
// the pipeline): a range [t, t1) of the pooled contexts walked through the chunk table (blocks
// stop at chunk ends, no mask), or a plain segment (the prefix, no mask) followed by a causal
// segment (self KV / own chunk).
struct Walk {
    // context mode (cu != NULL); the tables are read with scalar loads, once per chunk
    const int32_t* cu;
    const void* const* k_chunks;
    const void* const* v_chunks;
    const char *kbase, *vbase;       // rows of the current chunk for this KV head
    int n_chunks, c;
    int t, t1, c0, c1;
    long head_b;
    // sequence mode
    const char *kp, *vp, *kc, *vc;
    int np, nc, j, phase;
    long stride_b;

    __device__ void load_chunk() {
        kbase = (const char*)scalar_load_ptr(k_chunks + c) + head_b;
        vbase = (const char*)scalar_load_ptr(v_chunks + c) + head_b;
    }
    __device__ void init_ctx(const KvView& kv, long t0_, long t1_, long stride_b_, long head_b_) {
        cu = kv.cu; k_chunks = kv.k_chunks; v_chunks = kv.v_chunks; n_chunks = kv.n_chunks;
        t = (int)t0_; t1 = (int)t1_; stride_b = stride_b_; head_b = head_b_;
        c = 0; c0 = 0; c1 = 0; kbase = vbase = nullptr;
        kp = vp = kc = vc = nullptr; np = nc = j = 0; phase = 2;
        if (t < t1 && cu != nullptr) {
            int lo = 0, hi = n_chunks - 1;
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (scalar_load_i32(cu + mid) <= t) lo = mid; else hi = mid - 1;
            }
            c = lo; c0 = scalar_load_i32(cu + c); c1 = scalar_load_i32(cu + c + 1);
            load_chunk();
        } else {
            t1 = t;
        }
    }
    __device__ void init_seq(const char* kp_, const char* vp_, int np_, const char* kc_, const char* vc_, int nc_, long stride_b_) {
        cu = nullptr; k_chunks = v_chunks = nullptr; kbase = vbase = nullptr; n_chunks = c = 0; t = t1 = c0 = c1 = 0; head_b = 0;
        kp = kp_; vp = vp_; np = np_; kc = kc_; vc = vc_; nc = nc_; stride_b = stride_b_;
        j = 0; phase = np > 0 ? 0 : 1;
    }
    __device__ bool next(Block& b) {
        if (cu != nullptr) {
            if (t >= t1) return false;
            if (t >= c1) {
                do {                                                   // next non-empty chunk
                    if (c + 1 >= n_chunks) { t = t1; return false; }   // table shorter than total_ctx: stop, stay in bounds
                    ++c; c0 = c1; c1 = scalar_load_i32(cu + c + 1);
                } while (t >= c1);
                load_chunk();
            }
            const int e = c1 < t1 ? c1 : t1;
            const int n = e - t < BLK ? e - t : BLK;
            b.k = kbase + (long)(t - c0) * stride_b;
            b.v = vbase + (long)(t - c0) * stride_b;
            b.n_valid = n; b.j0 = -1;
            t += n;
            return true;
        }
        if (phase == 0) {
            const int n = np - j < BLK ? np - j : BLK;
            b.k = kp + (long)j * stride_b; b.v = vp + (long)j * stride_b; b.n_valid = n; b.j0 = -1;
            j += n;
            if (j >= np) { phase = 1; j = 0; }
            return true;
        }
        if (phase != 1 || j >= nc) return false;
        const int n = nc - j < BLK ? nc - j : BLK;
        b.k = kc + (long)j * stride_b; b.v = vc + (long)j * stride_b; b.n_valid = n; b.j0 = j;
        j += n;
        return true;
    }
};

// LDS layout of a block: K row r at r*256, 16-byte chunk index XOR (r & 15) (conflict-free 16-byte
// reads down a column of rows); V row r at 8192 + r*256, chunk index XOR 4*(r & 3) (the four rows
// of one transposing read land in distinct 64-byte windows).
//
// Direct global->LDS loads write lane i's 16 bytes at (wave-uniform LDS base) + 16*i, so one
// instruction fills four consecutive 256-byte rows; the swizzle is applied on the global side:
// lane i = (row r = i/16, physical chunk c = i%16) fetches logical chunk c ^ f(r).
// Wavefront w fills rows 8w .. 8w+7 of K and of V: four instructions per block.
// Rows past n_valid re-read the last valid row: finite data whose probabilities are zero.
struct LoadOffsets { uint32_t k[2], v[2]; };          // byte offsets of this lane's pieces from a block's row 0

__device__ __forceinline__ LoadOffsets load_offsets(long stride_b, int n_valid) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, rl = lane >> 4;
    LoadOffsets o;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int r = 8 * wave + 4 * i + rl;
        const int rr = r < n_valid ? r : n_valid - 1;
        o.k[i] = (uint32_t)rr * (uint32_t)stride_b + ((c ^ (r & 15)) << 4);
        o.v[i] = (uint32_t)rr * (uint32_t)stride_b + ((c ^ ((r & 3) << 2)) << 4);
    }
    return o;
}

// `full` holds the offsets of a full block (computed once); a partial block recomputes them with
// its rows clamped.  The block's base pointers are wavefront-uniform, the offsets 32-bit per lane.
__device__ __forceinline__ void issue_block_loads(const Block& b, long stride_b, char* slot, const LoadOffsets& full) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    LoadOffsets o = full;
    if (b.n_valid < BLK) o = load_offsets(stride_b, b.n_valid);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        char* dst = slot + (8 * wave + 4 * i) * ROWB;
        __builtin_amdgcn_global_load_lds((glb_void*)(b.k + o.k[i]), (lds_void*)dst, 16, 0, 0);
        __builtin_amdgcn_global_load_lds((glb_void*)(b.v + o.v[i]), (lds_void*)(dst + KVB), 16, 0, 0);
    }
}

// s_waitcnt vmcnt(n) only (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[15:14]).
// The direct-to-LDS loads complete in issue order; `blocks_younger` blocks may stay in flight.
__device__ __forceinline__ void wait_vmcnt(int blocks_younger) {
    if (blocks_younger >= 3) __builtin_amdgcn_s_waitcnt(0x0f70 | (3 * LOADS_PER_BLOCK));
    else if (blocks_younger == 2) __builtin_amdgcn_s_waitcnt(0x0f70 | (2 * LOADS_PER_BLOCK));
    else if (blocks_younger == 1) __builtin_amdgcn_s_waitcnt(0x0f70 | LOADS_PER_BLOCK);
    else __builtin_amdgcn_s_waitcnt(0x0f70);
}

// Workgroup barrier that the compiler may not move memory operations across, without the
// vmcnt(0) drain a fence would add (the loads in flight target other ring slots).
__device__ __forceinline__ void ring_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// The transposing LDS read.  The pointer is passed through a restrict-qualified parameter on
// purpose: once inlined, the read carries alias-scope information, like the plain K reads carry
// type information.  The compiler's wait-count pass drains ALL outstanding global->LDS loads
// before an LDS read it knows nothing about -- which would serialise the ring -- and leaves
// reads with alias information to the explicit wait_vmcnt()/barrier protocol below.
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
__device__ __forceinline__ s16x4 lds_read_tr_raw(lds_s16x4* __restrict__ p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(p);
}
__device__ __forceinline__ bf16x4 lds_read_tr(const char* p) {
    return __builtin_bit_cast(bf16x4, lds_read_tr_raw((lds_s16x4*)p));
}

// max over the two half-wavefronts (query row = lane & 31 lives in lanes l and l ^ 32)
__device__ __forceinline__ float max_halves(float x) {
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Per-wavefront state of RB blocks of 32 query rows.
template <int RB>
struct WaveState {
    float m[RB];                 // reference maximum, log2 units (score * scale * log2 e)
    float l[RB];                 // this lane's share of the running sum
    f32x16 o[RB][4];             // O^T accumulators: [row block][32-dim block]
};

// per-lane LDS byte offsets inside a slot (constant over the loop)
struct LaneOffsets {
    int k;                       // K fragment for k-slab ks: k ^ (32*ks)
    int v[4];                    // V^T fragment for dim block db; + 4096*sl + 2048*half
};

__device__ __forceinline__ LaneOffsets lane_offsets() {
    const int lane = threadIdx.x & 63;
    const int l32 = lane & 31, hi = lane >> 5, g16 = lane >> 4, s16 = lane & 15;
    LaneOffsets o;
    // A operand of K Q^T: token row l32, dims 16*ks + 8*hi .. +7 = chunk 2*ks + hi
    o.k = l32 * ROWB + ((hi ^ (l32 & 15)) << 4);
    // A operand of V^T P^T via the transposing read: this lane supplies the address of token row
    // 16*sl + 4*(g16 >> 1) + (s16 >> 2) (+8 for the second half), dims 32*db + 16*(g16 & 1) + 4*(s16 & 3) .. +3
    const int row0 = 4 * (g16 >> 1) + (s16 >> 2);
    const int chlow = 2 * (g16 & 1) + ((s16 & 3) >> 1);
#pragma unroll
    for (int db = 0; db < 4; ++db)
        o.v[db] = KVB + row0 * ROWB + (((4 * db + chlow) ^ ((row0 & 3) << 2)) << 4) + (s16 & 1) * 8;
    return o;
}

// S^T = K Q^T for one block (both row blocks share each K fragment).
template <int RB>
__device__ __forceinline__ void scores(const char* slot, const LaneOffsets& lo, const bf16x8 (&qf)[RB][8], f32x16 (&s)[RB]) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[rb][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 a = *(const bf16x8*)(slot + (lo.k ^ (32 * ks)));
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
            s[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[rb][ks], s[rb], 0, 0, 0);
    }
}

// O^T += V^T P^T for one block.  k-slot e of lane half `hi` in slab sl is token
// 16*sl + (e < 4 ? 4*hi + e : 8 + 4*hi + e - 4): two transposing reads per fragment.
template <int RB>
__device__ __forceinline__ void accumulate(const char* slot, const LaneOffsets& lo, const bf16x8 (&p)[RB][2], WaveState<RB>& st) {
#pragma unroll
    for (int sl = 0; sl < 2; ++sl)
#pragma unroll
        for (int db = 0; db < 4; ++db) {
            const bf16x4 lo4 = lds_read_tr(slot + lo.v[db] + 4096 * sl);
            const bf16x4 hi4 = lds_read_tr(slot + lo.v[db] + 4096 * sl + 2048);
            const bf16x8 a = __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
                st.o[rb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p[rb][sl], st.o[rb][db], 0, 0, 0);
        }
}

// Masks of a block (tail, causal diagonal); accumulator register r holds token
// 8*(r/4) + 4*hi + (r%4) of the block for query row lane & 31.
template <int RB>
__device__ __forceinline__ void apply_mask(f32x16 (&s)[RB], const Block& b, const int (&lim)[RB]) {
    const int hi = (threadIdx.x & 63) >> 5;
    // keep the vector writes below clear of the matrix-core writes to the same registers
    asm volatile("s_nop 15");
    asm volatile("s_nop 15");
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        // tokens of the block this row sees: [0, nvis)
        const int nvis = b.j0 >= 0 ? min(b.n_valid, lim[rb] - b.j0 + 1) : b.n_valid;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int tok = 8 * (r >> 2) + 4 * hi + (r & 3);
            s[rb][r] = tok < nvis ? s[rb][r] : -INFINITY;      // a select, not a branch
        }
    }
}

// ---- online softmax with a lazily maintained reference --------------------------------------
// Probabilities are taken against a per-row reference m (log2 units): p = 2^(s*sc2 - m).  fp32 and
// bf16 both carry 8 exponent bits, so m need not be the running maximum: any m within 2^kLazy of
// it loses no precision.  The fast path therefore never computes a maximum; it only checks,
// from the row sums it needs anyway, that no probability left the safe range -- or that a row
// whose reference is still unset (-inf) has just seen its first keys -- and in that rare case
// runs set_reference(), which takes the true row maxima, rescales O and l, and redoes the block.
__device__ __forceinline__ float max16(const f32x16& s) {
    return fmaxf(fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7]))),
                 fmaxf(fmaxf(fmaxf(s[8], s[9]), fmaxf(s[10], s[11])), fmaxf(fmaxf(s[12], s[13]), fmaxf(s[14], s[15]))));
}

// Two scores -> two bf16 probabilities (register pair k of row block rb).  The row sum is taken
// over the ROUNDED probabilities, the ones the PV product uses.
template <int RB>
__device__ __forceinline__ void softmax_pair(const f32x16 (&s)[RB], int rb, int k, float sc2, float m_use,
                                             float (&psum)[RB], bf16x8 (&p)[RB][2]) {
    const int r = 2 * k;
    const float p0 = __builtin_amdgcn_exp2f(fmaf(s[rb][r], sc2, -m_use));
    const float p1 = __builtin_amdgcn_exp2f(fmaf(s[rb][r + 1], sc2, -m_use));
    bf16x2 pk;
    pk[0] = (__bf16)p0; pk[1] = (__bf16)p1;
    const bf16x2 ones = {(__bf16)1.f, (__bf16)1.f};
#ifdef APE_X_NOSOFTMAX
    if (k) return;
#endif
    psum[rb] = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, psum[rb], false);
    p[rb][r >> 3][r & 7] = pk[0];
    p[rb][r >> 3][(r & 7) + 1] = pk[1];
}

__device__ __forceinline__ float ref_use(float m) { return m == -INFINITY ? 0.f : m; }

// O *= alpha (per query row).  The file is built with VGPR-form MFMAs (accumulators in the
// vector registers), so this is a plain multiply; it is kept clear of the matrix-core writes.
template <int RB>
__device__ __forceinline__ void rescale(WaveState<RB>& st, const float (&alpha)[RB]) {
    asm volatile("s_nop 15\n\ts_nop 15");
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) st.o[rb][db][r] *= alpha[rb];
    asm volatile("s_nop 7");
}

__device__ __forceinline__ bf16x8 read_k_frag(const char* slot, const LaneOffsets& lo, int ks) {
#ifdef APE_X_NOKREAD
    { u32x4 w = {(unsigned)lo.k, (unsigned)ks, (unsigned)(size_t)slot, 1u}; return __builtin_bit_cast(bf16x8, w); }
#endif
    return *(const bf16x8*)(slot + (lo.k ^ (32 * ks)));
}
// V^T fragment f = sl*4 + db
__device__ __forceinline__ bf16x8 read_v_frag(const char* slot, const LaneOffsets& lo, int f) {
#ifdef APE_X_NOVREAD
    { u32x4 w = {(unsigned)lo.v[f & 3], (unsigned)f, (unsigned)(size_t)slot, 1u}; return __builtin_bit_cast(bf16x8, w); }
#endif
    const bf16x4 lo4 = lds_read_tr(slot + lo.v[f & 3] + 4096 * (f >> 2));
    const bf16x4 hi4 = lds_read_tr(slot + lo.v[f & 3] + 4096 * (f >> 2) + 2048);
    return __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
}

// Keeps a value (and with it the slice of vector work that produced it) at this point of the
// program: the scheduling barriers below order machine instructions, this orders the IR.
__device__ __forceinline__ void pin(float& x) { asm volatile("" : "+v"(x)); }

// Rare path of the lazy reference: take the true row maxima of the (masked) scores of the
// current block, move the references that are unset or too low, bring O and l to them, and
// recompute the block's probabilities.
template <int RB>
__device__ __forceinline__ void set_reference(const f32x16 (&s_cur)[RB], float sc2, WaveState<RB>& st,
                                              float (&psum)[RB], bf16x8 (&p)[RB][2]) {
    float alpha[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const float mx = max_halves(max16(s_cur[rb])) * sc2;
        const float m_old = st.m[rb];
        const float m_new = (m_old == -INFINITY || mx > m_old + kLazy) ? mx : m_old;
        alpha[rb] = m_old == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_old - m_new);     // O = l = 0 while unset
        st.m[rb] = m_new;
        st.l[rb] *= alpha[rb];
    }
    rescale<RB>(st, alpha);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        psum[rb] = 0.f;
        const float m_use = ref_use(st.m[rb]);
#pragma unroll
        for (int k = 0; k < 8; ++k) softmax_pair<RB>(s_cur, rb, k, sc2, m_use, psum, p);
    }
}

// One step of the software pipeline, for block j, entered with its (masked) scores in s_cur.
// It runs  K Q^T of block j+1 -> s_nxt  (matrix cores)  |  softmax of block j -> p     (vector ALUs)
// then     O += P V of block j          (matrix cores)  |  s_cur <- s_nxt
// as an interleaved instruction stream: an MFMA, then a slice of vector work, pinned by
// scheduling barriers.  Without a next block (have_nxt false) slot_nxt is any landed slot: the
// scores are computed and dropped.
template <int RB>
__device__ __forceinline__ void pipeline_step(const char* slot_cur, const char* slot_nxt, const LaneOffsets& lo,
                                              const bf16x8 (&qf)[RB][8], WaveState<RB>& st, float sc2,
                                              f32x16 (&s_cur)[RB], const Block& nb, bool nxt_masked, const int (&lim)[RB]) {
    // ---- first half: 8*RB MFMAs of K Q^T, 8*RB slices of the softmax
    f32x16 s_nxt[RB];
    bf16x8 p[RB][2];
    float psum[RB], m_use[RB];
    bf16x8 kf[8];
    kf[0] = read_k_frag(slot_nxt, lo, 0);
    kf[1] = read_k_frag(slot_nxt, lo, 1);
    kf[2] = read_k_frag(slot_nxt, lo, 2);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        psum[rb] = 0.f;
        m_use[rb] = ref_use(st.m[rb]);
#pragma unroll
        for (int r = 0; r < 16; ++r) s_nxt[rb][r] = 0.f;
    }
    // two slices ahead of the first MFMA cover the latency of the first fragment reads
    softmax_pair<RB>(s_cur, 0, 0, sc2, m_use[0], psum, p);
    softmax_pair<RB>(s_cur, 0, 1, sc2, m_use[0], psum, p);
    pin(psum[0]);
    __builtin_amdgcn_sched_barrier(0);
    bf16x8 vf[8];
#pragma unroll
    for (int n = 0; n < 8 * RB; ++n) {
        const int ks = n / RB, rb = n % RB;
        if (rb == 0 && ks + 3 < 8) kf[ks + 3] = read_k_frag(slot_nxt, lo, ks + 3);
        if (rb == 0 && ks == 5) vf[0] = read_v_frag(slot_cur, lo, 0);
        if (rb == 0 && ks == 6) vf[1] = read_v_frag(slot_cur, lo, 1);
        if (rb == 0 && ks == 7) vf[2] = read_v_frag(slot_cur, lo, 2);
#ifdef APE_X_NOMFMA
        s_nxt[rb][ks] += __builtin_bit_cast(f32x4, kf[ks])[0] * __builtin_bit_cast(f32x4, qf[rb][ks])[1];
#else
        s_nxt[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[rb][ks], s_nxt[rb], 0, 0, 0);
#endif
        __builtin_amdgcn_sched_barrier(0);
        const int slice = n + 2;                                     // (row block, register pair)
        if (slice < 8 * RB) {
            softmax_pair<RB>(s_cur, slice / 8, slice % 8, sc2, m_use[slice / 8], psum, p);
            pin(psum[slice / 8]);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    // ---- did every probability stay in range, and is every row that saw a key referenced?
    bool bad = false;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
        bad |= !(psum[rb] <= 0x1p40f) || (st.m[rb] == -INFINITY && psum[rb] > 0.f);
    if (__builtin_expect(__builtin_amdgcn_ballot_w64(bad) != 0, 0)) set_reference<RB>(s_cur, sc2, st, psum, p);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) st.l[rb] += psum[rb];

    // ---- second half: 8*RB MFMAs of O += P V; in their shadow the scores of block j+1 become s_cur
#pragma unroll
    for (int n = 0; n < 8 * RB; ++n) {
        const int f = n / RB, rb = n % RB;                           // fragment f = sl*4 + db
        if (rb == 0 && f + 3 < 8) vf[f + 3] = read_v_frag(slot_cur, lo, f + 3);
#ifdef APE_X_NOMFMA
        st.o[rb][f & 3][f] += __builtin_bit_cast(f32x4, vf[f])[0] * __builtin_bit_cast(f32x4, p[rb][f >> 2])[1];
#else
        st.o[rb][f & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[f], p[rb][f >> 2], st.o[rb][f & 3], 0, 0, 0);
#endif
        __builtin_amdgcn_sched_barrier(0);
        if (n < 4 * RB) {
            const int r2 = n / 4, part = n % 4;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float t = s_nxt[r2][4 * part + e];
                pin(t);
                s_cur[r2][4 * part + e] = t;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    if (__builtin_expect(nxt_masked, 0)) apply_mask<RB>(s_cur, nb, lim);   // block tails, the causal diagonal
}

// Streams every block of the walk `lw`.  Every wavefront of the workgroup
// executes the same barriers and the same instruction stream; causal blocks a wavefront's rows
// do not see are simply masked.
//   vis_lo smallest causal limit among this wavefront's rows (blocks up to it need no causal mask)
#ifdef APE_TIMING
#define APE_T(i) do { const unsigned long long t__ = __builtin_amdgcn_s_memtime(); tacc[i] += t__ - tlast; tlast = __builtin_amdgcn_s_memtime(); } while (0)
#else
#define APE_T(i) do { } while (0)
#endif

template <int RB>
__device__ __forceinline__ void run_blocks(Walk lw, long stride_b, char* lds, const bf16x8 (&qf)[RB][8],
                                           WaveState<RB>& st, float sc2, const int (&lim)[RB], int vis_lo, unsigned long long* tdbg = nullptr) {
#ifdef APE_TIMING
    unsigned long long tacc[6] = {0, 0, 0, 0, 0, 0};
    unsigned long long tlast = __builtin_amdgcn_s_memtime();
#endif
    const LaneOffsets lo = lane_offsets();
    const LoadOffsets full = load_offsets(stride_b, BLK);
    // Loads run RING-1 blocks ahead of the compute.  What the compute needs to know of a block
    // in flight (valid rows, causal index of row 0) waits in a small FIFO: entry i describes
    // block j+1+i at the top of step j; n_valid == 0 marks "no such block".
    constexpr int FIFO = RING - 2;
    int f_nv[FIFO], f_j0[FIFO];
    Block lb, cb;
    bool more = lw.next(cb);
    if (!more) return;
    issue_block_loads(cb, stride_b, lds, full);
    int issued = 1;                                   // blocks whose loads have been issued
#pragma unroll
    for (int i = 0; i < FIFO; ++i) {
        f_nv[i] = 0; f_j0[i] = -1;
        if (more) {
            more = lw.next(lb);
            if (more) {
                issue_block_loads(lb, stride_b, lds + (issued % RING) * SLOTB, full);
                ++issued;
                f_nv[i] = lb.n_valid; f_j0[i] = lb.j0;
            }
        }
    }

    f32x16 s_cur[RB];                                 // (masked) scores of block j
    auto masked = [&](int n_valid, int j0) { return n_valid < BLK || (j0 >= 0 && j0 + BLK - 1 > vis_lo); };

    // block 0: scores (its reference is set by the first step's check)
    wait_vmcnt(issued - 1);
    ring_barrier();
    scores<RB>(lds, lo, qf, s_cur);
    if (masked(cb.n_valid, cb.j0)) apply_mask<RB>(s_cur, cb, lim);

    APE_T(0);
    bool have_cur = true;
    for (int j = 0; have_cur; ++j) {
        // block j+1: pop its description
        Block nb;
        nb.k = nb.v = nullptr; nb.n_valid = f_nv[0]; nb.j0 = f_j0[0];
        const bool have_nxt = nb.n_valid > 0;
#pragma unroll
        for (int i = 0; i + 1 < FIFO; ++i) { f_nv[i] = f_nv[i + 1]; f_j0[i] = f_j0[i + 1]; }
        f_nv[FIFO - 1] = 0; f_j0[FIFO - 1] = -1;
        APE_T(1);
        if (have_nxt) {
            // block j+1 must have landed; every wavefront is then also done with block j-1's
            // slot, which the next loads overwrite
#ifndef APE_X_NOLOAD
            wait_vmcnt(issued - (j + 2));
#endif
            APE_T(2);
#ifndef APE_X_NOBARRIER
            ring_barrier();
#endif
            APE_T(3);
            if (more) {
                more = lw.next(lb);
                if (more) {
#ifndef APE_X_NOLOAD
                    issue_block_loads(lb, stride_b, lds + (issued % RING) * SLOTB, full);
#endif
                    ++issued;
                    f_nv[FIFO - 1] = lb.n_valid; f_j0[FIFO - 1] = lb.j0;
                }
            }
        }
        const char* slot_cur = lds + (j % RING) * SLOTB;
        const char* slot_nxt = have_nxt ? lds + ((j + 1) % RING) * SLOTB : slot_cur;
        APE_T(4);
        pipeline_step<RB>(slot_cur, slot_nxt, lo, qf, st, sc2, s_cur, nb, have_nxt && masked(nb.n_valid, nb.j0), lim);
        have_cur = have_nxt;
        APE_T(5);
    }
#ifdef APE_TIMING
    if (tdbg && threadIdx.x == 0 && blockIdx.x == 0)
        for (int i = 0; i < 6; ++i) tdbg[i] = tacc[i];
#endif
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
    Walk walk;
    float sc2 = inv_sqrt_d * LOG2E;
    int vis_lo = 0, vis_hi = 0;
    if (split < a.n_ctx_splits) {
        const long t0 = (long)split * a.ctx_split_len;
        const long t1 = min((long)kv.total_ctx, t0 + a.ctx_split_len);
        walk.init_ctx(kv, t0, t1, stride_b, head_b);
        sc2 = inv_sqrt_d / kv.temperature * LOG2E;
    } else {
        // rows of this workgroup see the causal segment up to the last valid row's limit
        const int wg_tok_hi = min((qtile * BM + BM - 1) / G, q_len - 1);
        walk.init_seq((const char*)kv.k_prefix + head_b, (const char*)kv.v_prefix + head_b, kv.prefix_len,
                      (const char*)kv.k_self + head_b, (const char*)kv.v_self + head_b, wg_tok_hi + causal_off + 1, stride_b);
        vis_lo = tok_lo + causal_off; vis_hi = tok_hi + causal_off;
    }
#ifdef APE_TIMING
    run_blocks<RB>(walk, stride_b, lds, qf, st, sc2, lim, vis_lo, (unsigned long long*)(a.part_lse + (long)60 * a.units_total));
#else
    run_blocks<RB>(walk, stride_b, lds, qf, st, sc2, lim, vis_lo);
#endif

    // ---- block result (Appendix C.1): normalised values + natural-log LogSumExp
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int R = qtile * BM + wave * 32 * RB + rb * 32 + l32;
        const int tok = R / G, g = R % G;
        const float lt = st.l[rb] + __shfl_xor(st.l[rb], 32);
        if (tok >= q_len) continue;
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
    Walk walk;
    walk.init_seq((const char*)a.k_prefix + head_b, (const char*)a.v_prefix + head_b, a.prefix_len,
              (const char*)a.k + (long)c0 * stride_b + head_b, (const char*)a.v + (long)c0 * stride_b + head_b,
              wg_tok_hi + 1, stride_b);
    run_blocks<RB>(walk, stride_b, lds, qf, st, 0.08838834764831845f * LOG2E, lim, tok_lo);

#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int R = qtile * BM + wave * 32 * RB + rb * 32 + l32;
        const int tok = R / G, g = R % G;
        const float lt = st.l[rb] + __shfl_xor(st.l[rb], 32);
        if (tok >= len) continue;
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

#ifdef APE_X_RB1
int flash_block_rows(int rows_per_kv_head) { return 128; }
#else
int flash_block_rows(int rows_per_kv_head) { return rows_per_kv_head > 128 ? 256 : 128; }
#endif

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
