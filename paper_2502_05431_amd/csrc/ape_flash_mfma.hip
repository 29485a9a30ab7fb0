// Matrix-core flash attention for gfx950 (bf16, head_dim 128): query prefill over the cached
// contexts (split over the keys), the decode step (the same kernel on a tile of which one wavefront has
// query rows and the other three only fetch: it is bound by HBM) and the block-diagonal causal encoding
// of the contexts.
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
//     compute; rows are 256 bytes and XOR-swizzled so that every LDS read is conflict-free (the wide
//     tile keeps K column-major instead: one address register, k-slabs as immediates);
//   - scores are computed TRANSPOSED, S^T = K Q^T: the accumulator layout then puts one query
//     row in one lane (and its partner lane +32), so the softmax row reductions are in-lane,
//     and the bf16 probabilities are already laid out as the B operand of O^T += V^T P^T;
//   - V^T fragments come from LDS through the transposing read ds_read_b64_tr_b16;
//   - the loop is software-pipelined over three blocks: one body runs O += P V of block j-1,
//     then K Q^T of block j+1 with the softmax of block j in the shadow of its MFMAs;
//   - the softmax keeps a lazily updated reference instead of a running maximum, so its fast
//     path is two exponentials, two adds and a conversion per pair of scores;
//   - stretches of full, unmasked blocks of one segment run a branch-free body (in the wide
//     tile, long stretches in groups of bodies whose ring slots are compile-time constants); segment
//     ends, partial blocks and the causal diagonal take a generic body with the same arithmetic;
//   - what bounds the block loop is the instruction issue of the one wavefront per SIMD (wide tile:
//     about 180 instructions next to every 32 MFMAs, 112 of them the softmax), so the code below
//     counts instructions: addresses as immediates, values carried instead of recomputed, the wait
//     state after a write of M0 filled with the next address step.
// The file is compiled with the MFMA accumulators in the vector registers (VGPR form).
#include "ape_internal.h"

#define APE_RING_FN __device__ __forceinline__
#define ape_ring_load_i32 ::ape::scalar_load_i32
#define ape_ring_load_ptr ::ape::scalar_load_ptr
#define ape_ring_load_chunk ::ape::scalar_load_chunk
#define ape_ring_find_chunk ::ape::find_chunk
#include "ape_ring.h"

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
constexpr int NT = 256;                      // threads per workgroup
constexpr int NW = NT / 64;                  // wavefronts
static_assert(ROWB == D * 2, "row bytes");
constexpr int LOADS_PER_BLOCK = 4;           // direct-to-LDS load instructions per wavefront per block
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr float kLazy = 40.f;                // a reference moves only when exceeded by 2^kLazy
constexpr float kUnset = -1.0e30f;           // reference of a row that has not seen a key yet
constexpr float kPsumMax = 0x1p40f;          // a lane's block sum above this: some probability left the safe range

// LDS slots of the ring (blocks j and j+1 in use, the others in flight), by row blocks per
// wavefront: the wide tile runs one workgroup per CU and looks further ahead; the narrow tile
// leaves room for two workgroups per CU, whose wavefronts fill each other's issue gaps.
template <int RB> struct Ring { static constexpr int slots = RB == 2 ? 6 : 5; };

// LDS layout of a block, two forms for K.
// Row-major (the narrow tile, and with it the bandwidth-bound decode): K row r at r*256, 16-byte
// chunk index XOR (r & 15) (conflict-free 16-byte reads down a column of rows).
// Column-major (the wide tile): chunk c of row r at (r >> 4)*4096 + c*256 + (r & 15)*16 -- the 16
// rows a fragment read touches per pass are 256 consecutive bytes (no conflicts, no swizzle), and the
// fragment of k-slab ks is at one per-lane offset + 512*ks, an immediate: ONE address register and one
// addition per body instead of eight of each (a wavefront's instruction issue is what bounds the
// block loop).  Its loads gather 64 bytes from each of 16 rows per instruction instead of whole rows,
// which costs streaming rate from HBM -- hence not for the decode.
// V row r at 8192 + r*256, chunk index XOR 4*(r & 3) (the four rows of one transposing read land in
// distinct 64-byte windows).
//
// Direct global->LDS loads write lane i's 16 bytes at (wave-uniform LDS base) + 16*i, so one
// instruction fills four consecutive 256-byte rows; the swizzle is applied on the global side:
// lane i = (row r = i/16, physical chunk c = i%16) fetches logical chunk c ^ f(r).
// Wavefront w fills rows 8w .. 8w+7 of K and of V: four instructions per block.
// Rows past n_valid re-read the last valid row: finite data whose probabilities are zero.
// NT: the loads carry the non-temporal hint (the block is read by this workgroup only and will not be
// read again: a decode step, a query of a few rows).  Streams at 6.5 instead of 6.1 TB/s; K/V that
// other workgroups re-read from L2 (the encode, a query of several row tiles) must not carry it.
template <bool NT, bool KCOL>
struct LoadOffsetsT {
    uint32_t k[2], v[2];                                  // byte offsets of this lane's pieces from a block's row 0
    int wave_dst;                                         // where in a slot's K (and V) part this wavefront's loads land; wavefront-uniform
    static constexpr bool nt = NT;                        // non-temporal loads
    static constexpr bool kcol = KCOL;                    // column-major K in LDS
    static_assert(!(NT && KCOL), "the column-major form gathers 64-byte pieces: not for streams bound by HBM");
};

// The thread index for a tile's set-up (lane offsets, load offsets, query addresses): a kernel that
// walks several tiles makes it opaque per tile, so that everything derived from it is recomputed
// per tile instead of being kept in registers across the whole walk (the compiler would hoist it
// all out of the tile loop, and the block loop has no registers to spare).  Inside the block loop
// the few uses of the thread index read threadIdx directly, as a one-tile kernel does.
__device__ __forceinline__ int tile_thread_index() {
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    return tid;
}

template <bool NT, bool KCOL>
__device__ __forceinline__ LoadOffsetsT<NT, KCOL> load_offsets(long stride_b, int n_valid, int tid) {
    const int lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, rl = lane >> 4;
    LoadOffsetsT<NT, KCOL> o;
    o.wave_dst = __builtin_amdgcn_readfirstlane(wave) * (8 * ROWB);   // (kept in a scalar register over the block loop)
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int r = 8 * wave + 4 * i + rl;
        const int rr = r < n_valid ? r : n_valid - 1;
        o.v[i] = (uint32_t)rr * (uint32_t)stride_b + ((c ^ ((r & 3) << 2)) << 4);
        if constexpr (!KCOL) {
            o.k[i] = (uint32_t)rr * (uint32_t)stride_b + ((c ^ (r & 15)) << 4);
        } else {
            // column-major K: the wavefront's load i fills LDS bytes 1024*(2*wave + i) .. +1023 of the K part, i.e.
            // rows 16*(wave >> 1) .. +15 of chunks 8*(wave & 1) + 4*i .. +3; lane = (chunk within those, row)
            const int rk = 16 * (wave >> 1) + (lane & 15);
            const int rrk = rk < n_valid ? rk : n_valid - 1;
            o.k[i] = (uint32_t)rrk * (uint32_t)stride_b + ((8 * (wave & 1) + 4 * i + (lane >> 4)) << 4);
        }
    }
    return o;
}

// One direct global->LDS load: every lane fetches 16 bytes at base + voff (base wavefront-uniform,
// voff per lane) and the wavefront's 1 KB lands at the wavefront-uniform LDS address lds_dst (M0).
// Written as instructions: the scalar-base addressing form costs no vector address arithmetic,
// and the compiler then does not track these loads, which is intended -- they are ordered against
// the LDS reads by the explicit vmcnt waits and barriers of the ring, not by the compiler, which
// could only wait for all of them.
template <bool NT>
__device__ __forceinline__ void dma16(const char* base, uint32_t voff, const char* lds_dst) {
    const uint32_t m0v = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)lds_dst;
    if constexpr (NT)
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt"
                     :: "v"(voff), "s"(base), "s"(m0v) : "m0");
    else
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                     :: "v"(voff), "s"(base), "s"(m0v) : "m0");
}

// The same load inside a chain of loads: M0 is taken from `m0v`, and the instruction that must stand
// between the write of M0 and the load (a wait state) is the addition that moves `m0v` on to the next
// load's LDS address -- no s_nop, and no separate address arithmetic per load.
template <bool NT, int DELTA>
__device__ __forceinline__ void dma16_chain(const char* base, uint32_t voff, uint32_t& m0v) {
    if constexpr (NT)
        asm volatile("s_mov_b32 m0, %0\n\ts_add_i32 %0, %0, %3\n\tglobal_load_lds_dwordx4 %1, %2 nt"
                     : "+s"(m0v) : "v"(voff), "s"(base), "n"(DELTA) : "m0", "scc");
    else
        asm volatile("s_mov_b32 m0, %0\n\ts_add_i32 %0, %0, %3\n\tglobal_load_lds_dwordx4 %1, %2"
                     : "+s"(m0v) : "v"(voff), "s"(base), "n"(DELTA) : "m0", "scc");
}

// Load i (0..3) of a block: wavefront w fills rows 8w + 4(i/2) .. +3 of V (i odd), and of K (i even) in the
// row-major form; in the column-major form the same 1 KB of the slot holds what load_offsets says.
template <class LO>
__device__ __forceinline__ void issue_block_load(int i, const char* bk, const char* bv, char* slot, const LO& o) {
    const char* dst = slot + o.wave_dst + 4 * (i >> 1) * ROWB;
    if ((i & 1) == 0) dma16<LO::nt>(bk, o.k[i >> 1], dst);
    else dma16<LO::nt>(bv, o.v[i >> 1], dst + KVB);
}
// Loads 0..3 of a block issued in this order, one per call, with `m0v` carried between the calls
// (set by load 0): K rows +0, V rows +0 (KVB further on), K rows +4, V rows +4.
template <class LO>
__device__ __forceinline__ void issue_block_load_chain(int i, const char* bk, const char* bv, char* slot, const LO& o, uint32_t& m0v) {
    if (i == 0) m0v = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)(slot + o.wave_dst);
    if (i == 0) dma16_chain<LO::nt, KVB>(bk, o.k[0], m0v);
    else if (i == 1) dma16_chain<LO::nt, 4 * ROWB - KVB>(bv, o.v[0], m0v);
    else if (i == 2) dma16_chain<LO::nt, KVB>(bk, o.k[1], m0v);
    else dma16_chain<LO::nt, 0>(bv, o.v[1], m0v);
}

// `full` holds the offsets of a full block (computed once); a partial block recomputes them with
// its rows clamped.
template <class LO>
__device__ __forceinline__ void issue_block_loads(const char* bk, const char* bv, int n_valid, long stride_b, char* slot,
                                                  const LO& full) {
    LO o = full;
    if (__builtin_expect(n_valid < BLK, 0)) o = load_offsets<LO::nt, LO::kcol>(stride_b, n_valid, threadIdx.x);
#pragma unroll
    for (int i = 0; i < LOADS_PER_BLOCK; ++i) issue_block_load(i, bk, bv, slot, o);
}

// Takes the stream's next block and starts its loads into `slot`.
template <class LO>
__device__ __forceinline__ int issue_next(Stream& ld, char* slot, const LO& full) {
    const char *bk, *bv;
    const int d = ld.take(bk, bv);
    issue_block_loads(bk, bv, desc_n(d), ld.stride_b, slot, full);
    return d;
}

// s_waitcnt vmcnt(n) only (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[15:14]).
// The direct-to-LDS loads complete in issue order, so "all but the youngest n blocks have
// landed" is vmcnt(n * LOADS_PER_BLOCK).
template <int BLOCKS_YOUNGER>
__device__ __forceinline__ void wait_blocks() {
    constexpr int n = BLOCKS_YOUNGER * LOADS_PER_BLOCK;
    static_assert(n < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0f70 | (n & 15) | ((n >> 4) << 14));
}

// Workgroup barrier that the compiler may not move memory operations across, without the
// vmcnt(0) drain a fence would add (the loads in flight target other ring slots).
__device__ __forceinline__ void ring_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

__device__ __forceinline__ bf16x4 lds_read_tr(const char* p) {
    s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
    return __builtin_bit_cast(bf16x4, r);
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
    int k;                       // K fragment for k-slab ks: k ^ (32*ks) (row-major), k + 512*ks (column-major)
    int v[4];                    // V^T fragment for dim block db; + 4096*sl + 2048*half
};

template <bool KCOL>
__device__ __forceinline__ LaneOffsets lane_offsets(int tid) {
    const int lane = tid & 63;
    const int l32 = lane & 31, hi = lane >> 5, g16 = lane >> 4, s16 = lane & 15;
    LaneOffsets o;
    // A operand of K Q^T: token row l32, dims 16*ks + 8*hi .. +7 = chunk 2*ks + hi
    if constexpr (KCOL) o.k = (l32 >> 4) * 4096 + hi * 256 + (l32 & 15) * 16;
    else o.k = l32 * ROWB + ((hi ^ (l32 & 15)) << 4);
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
template <int RB, bool KCOL>
__device__ __forceinline__ void scores(const char* slot, const LaneOffsets& lo, const bf16x8 (&qf)[RB][8], f32x16 (&s)[RB]) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[rb][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 a = *(const bf16x8*)(slot + (KCOL ? lo.k + 512 * ks : lo.k ^ (32 * ks)));
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
__device__ __forceinline__ void apply_mask(f32x16 (&s)[RB], int desc, const int (&lim)[RB]) {
    const int n_valid = desc_n(desc), j0 = desc_j0(desc);
    const int hi = (threadIdx.x & 63) >> 5;
    // keep the vector writes below clear of the matrix-core writes to the same registers
    asm volatile("s_nop 15");
    asm volatile("s_nop 15");
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        // tokens of the block this row sees: [0, nvis)
        const int nvis = j0 >= 0 ? min(n_valid, lim[rb] - j0 + 1) : n_valid;
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
// from the block sums it needs anyway, that no probability left the safe range.  A row that has
// not seen a key yet carries the reference kUnset, against which every finite score overflows,
// so its first keys trip the same check.  Then set_reference() takes the true row maxima,
// rescales O and l, and redoes the block's probabilities.
__device__ __forceinline__ float max16(const f32x16& s) {
    return fmaxf(fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7]))),
                 fmaxf(fmaxf(fmaxf(s[8], s[9]), fmaxf(s[10], s[11])), fmaxf(fmaxf(s[12], s[13]), fmaxf(s[14], s[15]))));
}

// The softmax of a block is cut into slices of two scores (register pair k of row block rb):
// two exponentials, their fp32 row sum, one packed conversion to bf16.  (The row sum is taken in
// plain fp32 adds on purpose: the bf16 dot-product instruction would do it in one instruction,
// but it does not overlap with a running MFMA, which these do.)  The conversion is written as an
// instruction so that it stays in its slice; it lists the new sums as inputs only to be ordered
// after them, which also keeps it clear of the exponentials it reads.
// p[rb][sl] holds the probabilities of k-slab sl as four packed pairs.
template <int RB>
__device__ __forceinline__ void softmax_slice(const f32x16 (&s)[RB], int rb, int k, float sc2, float m,
                                              float (&psum)[RB][2], u32x4 (&p)[RB][2]) {
    const int r = 2 * k;
    const float e0 = __builtin_amdgcn_exp2f(fmaf(s[rb][r], sc2, -m));
    const float e1 = __builtin_amdgcn_exp2f(fmaf(s[rb][r + 1], sc2, -m));
    // (The additions also keep the conversion below, which the compiler does not look into, one
    // instruction away from the exponentials: a vector instruction that reads a transcendental's result
    // in the very next issue slot gets a stale value.  Starting the sums by assignment in slice 0 saved
    // two instructions per row block and produced exactly that.)
    psum[rb][0] += e0;
    psum[rb][1] += e1;
    uint32_t pk;
    asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(pk) : "v"(e0), "v"(e1), "v"(psum[rb][0]), "v"(psum[rb][1]));
    p[rb][r >> 3][(r & 7) >> 1] = pk;
}

// The same slice cut in two, for bodies that spread the softmax over every MFMA slot: first the two
// exponentials (their arguments are ready since the previous body), then, one MFMA later, the row
// sums and the packed conversion.
template <int RB>
__device__ __forceinline__ void softmax_half_a(const f32x16 (&s)[RB], int rb, int k, float sc2, float m, float (&e)[2]) {
    e[0] = __builtin_amdgcn_exp2f(fmaf(s[rb][2 * k], sc2, -m));
    e[1] = __builtin_amdgcn_exp2f(fmaf(s[rb][2 * k + 1], sc2, -m));
}
template <int RB>
__device__ __forceinline__ void softmax_half_b(const float (&e)[2], int rb, int k, float (&psum)[RB][2], u32x4 (&p)[RB][2]) {
    const int r = 2 * k;
    psum[rb][0] += e[0];
    psum[rb][1] += e[1];
    uint32_t pk;
    asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(pk) : "v"(e[0]), "v"(e[1]), "v"(psum[rb][0]), "v"(psum[rb][1]));
    p[rb][r >> 3][(r & 7) >> 1] = pk;
}

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

template <bool KCOL>
__device__ __forceinline__ bf16x8 read_k_frag(const char* slot, const LaneOffsets& lo, int ks) {
    if constexpr (KCOL) return *(const bf16x8*)(slot + lo.k + 512 * ks);
    else return *(const bf16x8*)(slot + (lo.k ^ (32 * ks)));
}
// V^T fragment f = sl*4 + db
__device__ __forceinline__ bf16x8 read_v_frag(const char* slot, const LaneOffsets& lo, int f) {
    const bf16x4 lo4 = lds_read_tr(slot + lo.v[f & 3] + 4096 * (f >> 2));
    const bf16x4 hi4 = lds_read_tr(slot + lo.v[f & 3] + 4096 * (f >> 2) + 2048);
    return __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
}
// The narrow tile keeps the lane's four V^T addresses (slot + lane offset, one per dim block) from body
// to body: a block's fragments are read in two bodies (tokens 0..15 while it is block j, tokens 16..31
// while it is block j-1), and one addition per dim block moves an address on to the next block's slot
// -- four additions per body instead of eight.  (CARRY false, the wide tile: the same change made the
// compiler shuffle a hundred values per body through the accumulation registers; it adds slot and
// lane offset at every read and leaves `va` alone.)
struct VAddr { const char* a[4]; };
template <bool CARRY>
__device__ __forceinline__ bf16x8 read_v_pv(const VAddr& va, const char* slot_pv, const LaneOffsets& lo, int f) {
    if constexpr (!CARRY) return read_v_frag(slot_pv, lo, f);
    const bf16x4 lo4 = lds_read_tr(va.a[f & 3] + 4096 * (f >> 2));
    const bf16x4 hi4 = lds_read_tr(va.a[f & 3] + 4096 * (f >> 2) + 2048);
    return __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
}
template <bool CARRY>
__device__ __forceinline__ bf16x8 read_v_cur(VAddr& va, const char* slot_cur, const char* slot_pv, const LaneOffsets& lo, int f) {
    if constexpr (!CARRY) return read_v_frag(slot_cur, lo, f);
    va.a[f] += slot_cur - slot_pv;                                   // (f < 4: the dim block)
    const bf16x4 lo4 = lds_read_tr(va.a[f]);
    const bf16x4 hi4 = lds_read_tr(va.a[f] + 2048);
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
                                              float (&psum)[RB][2], u32x4 (&p)[RB][2]) {
    float alpha[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const float mx = max_halves(max16(s_cur[rb])) * sc2;             // -inf: the row sees nothing here
        const float m_old = st.m[rb];
        const float m_new = mx > m_old + kLazy ? mx : m_old;             // (kUnset + kLazy == kUnset)
        alpha[rb] = __builtin_amdgcn_exp2f(m_old - m_new);               // unset -> set: 0, and O = l = 0 anyway
        st.m[rb] = m_new;
        st.l[rb] *= alpha[rb];
    }
    rescale<RB>(st, alpha);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        psum[rb][0] = psum[rb][1] = 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) softmax_slice<RB>(s_cur, rb, k, sc2, st.m[rb], psum, p);
        psum[rb][0] += psum[rb][1];                                      // the caller adds [0] to l
    }
}

__device__ __forceinline__ float vmov(float x) {
    float y;
    asm volatile("v_mov_b32 %0, %1" : "=v"(y) : "v"(x));
    return y;
}

// One body of the software pipeline.  Entered with the raw scores of block j in s_b, the
// probabilities of block j-1 in p and its first V^T fragments in vf[0..3]; it runs
//     O += P V of block j-1     (matrix cores)  |  s_a <- s_b, K fragments of block j+1, the loads
//                                                  of the new block, ring bookkeeping
//     K Q^T of block j+1 -> s_b (matrix cores)  |  softmax of block j (s_a) -> p, V^T fragments of block j
// as an interleaved instruction stream: an MFMA, then a slice of other work, pinned by scheduling
// barriers.  What matters is the number of instructions per MFMA, and that they sit between the
// MFMAs.  The body starts with the PV product because that needs nothing of the block that has
// just landed: the latency of the first K fragment reads hides behind it.  Without a next block
// (d_nxt == 0) the scores are computed from a landed slot and dropped.  (Making these MFMAs
// conditional costs more than it saves: the accumulators then pass through copies.)
// On return the plan describes the next body.
template <int RB, int RING, bool FAST, class LO>
__device__ __forceinline__ void pipeline_body(char* lds, int pv_off, const LaneOffsets& lo, const LO& full,
                                              const bf16x8 (&qf)[RB][8], WaveState<RB>& st, float sc2,
                                              f32x16 (&s_b)[RB], u32x4 (&p)[RB][2], bf16x8 (&vf)[8], VAddr& va,
                                              RingPlan<RING>& plan, const int (&lim)[RB]) {
    constexpr int NS = 8 * RB;                                       // MFMAs per half
    const int d_cur = plan.d_cur, d_nxt = FAST ? BLK : plan.d_nxt;
    const bool cur_masked = !FAST && plan.cur_masked;
    const char* slot_pv = lds + pv_off;
    const char* slot_cur = lds + plan.o_cur;
    const char* slot_nxt = lds + (d_nxt != 0 ? plan.o_nxt : plan.o_cur);

    // ---- first half: NS MFMAs of O += P V.  Its slices: first the LDS reads (the other V^T
    // fragments of block j-1, the K fragments of block j+1 -- each several MFMAs ahead of its
    // use), the new block's loads and the ring bookkeeping; then s_a <- s_b.
    f32x16 s_a[RB];
    bf16x8 kf[8];
    uint32_t m0v = 0;                                             // LDS address of the next load of the new block (see issue_block_load_chain)
#pragma unroll
    for (int n = 0; n < NS; ++n) {
        const int f = n / RB, rb = n % RB;                           // fragment f = sl*4 + db
        st.o[rb][f & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[f], __builtin_bit_cast(bf16x8, p[rb][f >> 2]),
                                                                  st.o[rb][f & 3], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (n < 2) {
            vf[4 + 2 * n] = read_v_pv<RB == 1>(va, slot_pv, lo, 4 + 2 * n);
            vf[5 + 2 * n] = read_v_pv<RB == 1>(va, slot_pv, lo, 5 + 2 * n);
        }
        if (RB == 2) {                                               // K fragments: slices 2, 3, 4
            if (n == 2) { kf[0] = read_k_frag<LO::kcol>(slot_nxt, lo, 0); kf[1] = read_k_frag<LO::kcol>(slot_nxt, lo, 1); kf[2] = read_k_frag<LO::kcol>(slot_nxt, lo, 2); }
            if (n == 3) { kf[3] = read_k_frag<LO::kcol>(slot_nxt, lo, 3); kf[4] = read_k_frag<LO::kcol>(slot_nxt, lo, 4); kf[5] = read_k_frag<LO::kcol>(slot_nxt, lo, 5); }
            if (n == 4) { kf[6] = read_k_frag<LO::kcol>(slot_nxt, lo, 6); kf[7] = read_k_frag<LO::kcol>(slot_nxt, lo, 7); }
        } else {                                                     // ... after the wait for the V^T fragments: slices 4, 5
            if (n == 4 || n == 5) {
#pragma unroll
                for (int q = 0; q < 4; ++q) kf[4 * (n - 4) + q] = read_k_frag<LO::kcol>(slot_nxt, lo, 4 * (n - 4) + q);
            }
        }
        if (FAST) {
            if (n < LOADS_PER_BLOCK) issue_block_load_chain(n, plan.new_k, plan.new_v, lds + plan.o_new, full, m0v);
            else
            if (n < LOADS_PER_BLOCK + 3) plan.fast_piece(n - LOADS_PER_BLOCK);
        } else if (n == 0) {
            if (plan.d_new != 0)
                issue_block_loads(plan.new_k, plan.new_v, desc_n(plan.d_new), plan.ld.stride_b, lds + plan.o_new, full);
        } else if (d_nxt != 0) {
            plan.piece(n - 1);                                       // (a uniform branch; nothing to plan after the last block)
        }
        if (n >= NS - 4 * RB) {                                      // the last 4*RB slices: four scores each
            const int c = n - (NS - 4 * RB), r2 = c / 4, part = c % 4;
#pragma unroll
            for (int q = 0; q < 4; ++q) s_a[r2][4 * part + q] = vmov(s_b[r2][4 * part + q]);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    if (__builtin_expect(cur_masked, 0)) apply_mask<RB>(s_a, d_cur, lim);   // block tails, the causal diagonal

    // ---- second half: NS MFMAs of K Q^T, each followed by a slice of the softmax
    float psum[RB][2];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        psum[rb][0] = psum[rb][1] = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) s_b[rb][r] = 0.f;
    }
#pragma unroll
    for (int n = 0; n < NS; ++n) {
        const int ks = n / RB, rb = n % RB;
        s_b[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[rb][ks], s_b[rb], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        softmax_slice<RB>(s_a, n / 8, n % 8, sc2, st.m[n / 8], psum, p);
        if (n < 4) vf[n] = read_v_cur<RB == 1>(va, slot_cur, slot_pv, lo, n);   // for the next body's PV
        __builtin_amdgcn_sched_barrier(0);
    }
    // ---- did every probability stay in range?  (kUnset rows that saw a key did not)
    bool bad = false;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        psum[rb][0] += psum[rb][1];
        bad |= !(psum[rb][0] <= kPsumMax);
    }
    if (__builtin_expect(__builtin_amdgcn_ballot_w64(bad) != 0, 0)) set_reference<RB>(s_a, sc2, st, psum, p);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) st.l[rb] += psum[rb][0];
}

// The fast body again, for pairs of bodies: it reads the scores of block j from s_in and writes
// those of block j+1 to s_out, two different register sets that swap roles from one body to the
// next, so no score is ever copied and the softmax is free to sit in either half.  With two row
// blocks it is dealt over the MFMA slots in half-slices, behind the PV MFMAs that still read the
// probabilities of block j-1 (see wide_half_slice below; measured against whole slices in the sixteen
// middle slots: config-3 prefill 0.508 -> 0.4925 ms, 16384-token chunks' encode 15.29 -> 14.65 ms);
// with one row block its first four slices run in the last four of the PV half.
template <int RB, int RING, class LO, int PH = -1>
__device__ __forceinline__ void pipeline_body_pp(char* lds, int pv_off, const LaneOffsets& lo, const LO& full,
                                                 const bf16x8 (&qf)[RB][8], WaveState<RB>& st, float sc2,
                                                 const f32x16 (&s_in)[RB], f32x16 (&s_out)[RB], u32x4 (&p)[RB][2],
                                                 bf16x8 (&vf)[8], VAddr& va, RingPlan<RING>& plan) {
    constexpr int NS = 8 * RB;
    // PH >= 0: block j sits in ring slot PH, known at compile time (the slot offsets then fold into
    // the LDS instructions' offset fields); the ring offsets of the plan stay where they are (see run_blocks)
    constexpr bool STATIC = PH >= 0;
    const char* slot_pv = STATIC ? lds + ((PH + RING - 1) % RING) * SLOTB : lds + pv_off;
    const char* slot_cur = STATIC ? lds + (PH % RING) * SLOTB : lds + plan.o_cur;
    const char* slot_nxt = STATIC ? lds + ((PH + 1) % RING) * SLOTB : lds + plan.o_nxt;
    char* slot_new = STATIC ? lds + ((PH + RING - 2) % RING) * SLOTB : lds + plan.o_new;
    bf16x8 kf[8];
    uint32_t m0v = 0;                                             // LDS address of the next load of the new block (see issue_block_load_chain)
    float psum[RB][2];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) psum[rb][0] = psum[rb][1] = 0.f;
    // Wide tile: the softmax in half-slices (two exponentials; then, a slot later, the sums and the
    // conversion), one per MFMA slot from slot 2 on, so that no slot carries more vector work than its MFMA
    // covers.  The probabilities of block j overwrite those of block j-1 as the PV MFMAs let go of them: the
    // MFMAs of slots 0..3 read p[0][0], 4..7 p[0][1], 8..11 p[1][0], 12..15 p[1][1], and slice i = (row block
    // i / 8, register pair i % 8) writes p[i / 8][(i % 8) / 4] in slot 2 i + 3 or later.
    float e_half[2];
    auto wide_half_slice = [&](int t) {                              // t = 0 .. 31: half-slice t
        const int i = t >> 1, rb = i / 8, k = i % 8;
        if ((t & 1) == 0) softmax_half_a<RB>(s_in, rb, k, sc2, st.m[rb], e_half);
        else softmax_half_b<RB>(e_half, rb, k, psum, p);
    };
    auto wide_slot = [&](int n) {                                    // n = 0 .. 31: the MFMA slot
        if (n < 2) return;
        if (n < 30) wide_half_slice(n - 2);
        else { wide_half_slice(2 * n - 32); wide_half_slice(2 * n - 31); }   // slots 30, 31: two each
    };
    // ---- O += P V of block j-1
#pragma unroll
    for (int n = 0; n < NS; ++n) {
        const int rb = n / 8, f = n % 8;                             // row block 0 first
        st.o[rb][f & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[f], __builtin_bit_cast(bf16x8, p[rb][f >> 2]),
                                                                  st.o[rb][f & 3], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (RB == 2) {
            // one fragment per slot: V^T fragments 4..7 of block j-1 in slots 0..3 (each used four slots later),
            // K fragments 0..3 of block j+1 in slots 4..7 (the fragments of k-slabs 4..7 are read in the K Q^T
            // half, when the scores of block j are mostly consumed: sixteen registers fewer at the body's
            // fullest point)
            if (n < 4) vf[4 + n] = read_v_pv<RB == 1>(va, slot_pv, lo, 4 + n);
            else if (n < 8) kf[n - 4] = read_k_frag<LO::kcol>(slot_nxt, lo, n - 4);
        } else if (n < 2) {
            vf[4 + 2 * n] = read_v_pv<RB == 1>(va, slot_pv, lo, 4 + 2 * n);
            vf[5 + 2 * n] = read_v_pv<RB == 1>(va, slot_pv, lo, 5 + 2 * n);
        } else if (n == 4 || n == 5) {                               // (after the wait for the V^T fragments)
#pragma unroll
            for (int q = 0; q < 4; ++q) kf[4 * (n - 4) + q] = read_k_frag<LO::kcol>(slot_nxt, lo, 4 * (n - 4) + q);
        }
        if (n < LOADS_PER_BLOCK) issue_block_load_chain(n, plan.new_k, plan.new_v, slot_new, full, m0v);
        else if (n < LOADS_PER_BLOCK + (STATIC ? 2 : 3)) plan.fast_piece(n - LOADS_PER_BLOCK);   // (piece 2 turns the ring offsets)
        if (RB == 2) wide_slot(n);
        if (RB == 1 && n >= 4) softmax_slice<RB>(s_in, 0, n - 4, sc2, st.m[0], psum, p);   // slab 0, last read by MFMA 3
        __builtin_amdgcn_sched_barrier(0);
    }
    // ---- K Q^T of block j+1, the rest of the softmax of block j
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s_out[rb][r] = 0.f;
#pragma unroll
    for (int n = 0; n < NS; ++n) {
        const int ks = n / RB, rb = n % RB;
        s_out[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[rb][ks], s_out[rb], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (RB == 2) wide_slot(NS + n);
        if (RB == 1 && n < 4) softmax_slice<RB>(s_in, 0, n + 4, sc2, st.m[0], psum, p);
        if (n < 4) vf[n] = read_v_cur<RB == 1>(va, slot_cur, slot_pv, lo, n);   // for the next body's PV
        if (RB == 2 && n >= 4 && n < 8) kf[n] = read_k_frag<LO::kcol>(slot_nxt, lo, n);   // first used by MFMA 8
        __builtin_amdgcn_sched_barrier(0);
    }
    bool bad = false;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        psum[rb][0] += psum[rb][1];
        bad |= !(psum[rb][0] <= kPsumMax);
    }
    if (__builtin_expect(__builtin_amdgcn_ballot_w64(bad) != 0, 0)) set_reference<RB>(s_in, sc2, st, psum, p);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) st.l[rb] += psum[rb][0];
}

// The fast body once more, with the softmax spread evenly: the probabilities of block j are written
// to p_out while the PV product still reads those of block j-1 from p_in (two register sets that
// swap roles from one body to the next, like the scores), so a slice of the softmax no longer has to
// wait for the MFMAs that read the registers it overwrites, and every one of the 16*RB MFMAs of the
// body carries half a slice (two exponentials, or two adds and a conversion) in its shadow instead
// of half of them carrying a whole one.
template <int RB, int RING, class LO>
__device__ __forceinline__ void pipeline_body_even(char* lds, int pv_off, const LaneOffsets& lo, const LO& full,
                                                   const bf16x8 (&qf)[RB][8], WaveState<RB>& st, float sc2,
                                                   const f32x16 (&s_in)[RB], f32x16 (&s_out)[RB],
                                                   const u32x4 (&p_in)[RB][2], u32x4 (&p_out)[RB][2],
                                                   bf16x8 (&vf)[8], VAddr& va, RingPlan<RING>& plan) {
    constexpr int NS = 8 * RB;
    const char* slot_pv = lds + pv_off;
    const char* slot_cur = lds + plan.o_cur;
    const char* slot_nxt = lds + plan.o_nxt;
    bf16x8 kf[8];
    uint32_t m0v = 0;                                             // LDS address of the next load of the new block (see issue_block_load_chain)
    float psum[RB][2];
    float e[2];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) psum[rb][0] = psum[rb][1] = 0.f;
    // slot t (0 .. 2*NS-1) carries half-slice t: slice t/2 = (row block (t/2)/8, register pair (t/2)%8)
    auto half_slice = [&](int t) {
        const int sl = t >> 1, rb = sl / 8, k = sl % 8;
        if ((t & 1) == 0) softmax_half_a<RB>(s_in, rb, k, sc2, st.m[rb], e);
        else softmax_half_b<RB>(e, rb, k, psum, p_out);
    };
    // ---- O += P V of block j-1
#pragma unroll
    for (int n = 0; n < NS; ++n) {
        const int rb = n / 8, f = n % 8;
        st.o[rb][f & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[f], __builtin_bit_cast(bf16x8, p_in[rb][f >> 2]),
                                                                  st.o[rb][f & 3], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (RB == 2) {
            if (n < 2) {
                vf[4 + 2 * n] = read_v_pv<RB == 1>(va, slot_pv, lo, 4 + 2 * n);
                vf[5 + 2 * n] = read_v_pv<RB == 1>(va, slot_pv, lo, 5 + 2 * n);
            }
            if (n == 2) { kf[0] = read_k_frag<LO::kcol>(slot_nxt, lo, 0); kf[1] = read_k_frag<LO::kcol>(slot_nxt, lo, 1); kf[2] = read_k_frag<LO::kcol>(slot_nxt, lo, 2); }
            if (n == 3) { kf[3] = read_k_frag<LO::kcol>(slot_nxt, lo, 3); kf[4] = read_k_frag<LO::kcol>(slot_nxt, lo, 4); kf[5] = read_k_frag<LO::kcol>(slot_nxt, lo, 5); }
            if (n == 4) { kf[6] = read_k_frag<LO::kcol>(slot_nxt, lo, 6); kf[7] = read_k_frag<LO::kcol>(slot_nxt, lo, 7); }
        } else {
            // narrow tile: the reads spread over the slots -- one V^T fragment of block j-1 in each of slots 0..3 (used
            // four slots later), two K fragments of block j+1 in each of slots 4..7
            if (n < 4) vf[4 + n] = read_v_pv<RB == 1>(va, slot_pv, lo, 4 + n);
            else { kf[2 * (n - 4)] = read_k_frag<LO::kcol>(slot_nxt, lo, 2 * (n - 4)); kf[2 * (n - 4) + 1] = read_k_frag<LO::kcol>(slot_nxt, lo, 2 * (n - 4) + 1); }
        }
        if (n < LOADS_PER_BLOCK) issue_block_load_chain(n, plan.new_k, plan.new_v, lds + plan.o_new, full, m0v);
        else if (n < LOADS_PER_BLOCK + 3) plan.fast_piece(n - LOADS_PER_BLOCK);
        half_slice(n);
        __builtin_amdgcn_sched_barrier(0);
    }
    // ---- K Q^T of block j+1
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s_out[rb][r] = 0.f;
#pragma unroll
    for (int n = 0; n < NS; ++n) {
        const int ks = n / RB, rb = n % RB;
        s_out[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[rb][ks], s_out[rb], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        half_slice(NS + n);
        if (n < 4) vf[n] = read_v_cur<RB == 1>(va, slot_cur, slot_pv, lo, n);   // for the next body's PV
        __builtin_amdgcn_sched_barrier(0);
    }
    bool bad = false;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        psum[rb][0] += psum[rb][1];
        bad |= !(psum[rb][0] <= kPsumMax);
    }
    if (__builtin_expect(__builtin_amdgcn_ballot_w64(bad) != 0, 0)) set_reference<RB>(s_in, sc2, st, psum, p_out);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) st.l[rb] += psum[rb][0];
}

// The loads of the first blocks of a stream (blocks 0 .. RING-3), started before anything else in
// the kernel -- the query fragments are fetched while they fly.
template <int RING, bool NT, bool KCOL = false>
struct RingStart {
    static constexpr int NF = RING - 3;
    RingPlan<RING> plan;
    LoadOffsetsT<NT, KCOL> full;
    int tid;                      // the tile's thread index (see tile_thread_index)
    int d0;
    int first[NF + 1];
};

template <int RING, bool NT, bool KCOL>
__device__ __forceinline__ void start_stream(RingStart<RING, NT, KCOL>& rs, const Stream& ld0, char* lds, int vis_lo, int tid) {
    constexpr int NF = RING - 3;
    rs.plan.ld = ld0;
    rs.plan.vis_lo = vis_lo;
    rs.full = load_offsets<NT, KCOL>(ld0.stride_b, BLK, tid);
    rs.tid = tid;
    rs.d0 = 0;
#pragma unroll
    for (int i = 0; i <= NF; ++i) rs.first[i] = 0;
    if (ld0.rem == 0) return;
    rs.d0 = issue_next(rs.plan.ld, lds, rs.full);
#pragma unroll
    for (int i = 0; i < NF; ++i) rs.first[i] = rs.plan.ld.rem > 0 ? issue_next(rs.plan.ld, lds + (i + 1) * SLOTB, rs.full) : 0;
}

// Streams every block through the ring.  Every wavefront of the workgroup executes the same
// barriers and the same instruction stream; causal blocks a wavefront's rows do not see are
// simply masked.  (vis_lo, given to start_stream: the smallest causal limit among this
// wavefront's rows; blocks up to it need no causal mask.)
// RING fast bodies, pair by pair, with block j of the first one in ring slot 0: every slot offset is a
// compile-time constant, so slot and lane offset of an LDS read need no addition (the slot goes into
// the instruction's offset field) and the loads' LDS addresses are constants plus the wavefront's share.
// The plan's ring offsets are not turned (after RING bodies they would be back where they are), and
// neither is the caller's pv_off.
template <int RB, int RING, int PH, class LO>
__device__ __forceinline__ void static_bodies(char* lds, const LaneOffsets& lo, const LO& full, const bf16x8 (&qf)[RB][8],
                                              WaveState<RB>& st, float sc2, f32x16 (&s_b)[RB], f32x16 (&s_c)[RB],
                                              u32x4 (&p)[RB][2], bf16x8 (&vf)[8], VAddr& va, RingPlan<RING>& plan) {
    constexpr int NF = RING - 3;
    static_assert(RING % 2 == 0, "pairs of bodies must tile the ring");
    if constexpr (PH < RING) {
        wait_blocks<NF - 1>(); ring_barrier();
        pipeline_body_pp<RB, RING, LO, PH>(lds, 0, lo, full, qf, st, sc2, s_b, s_c, p, vf, va, plan);
        wait_blocks<NF - 1>(); ring_barrier();
        pipeline_body_pp<RB, RING, LO, PH + 1>(lds, 0, lo, full, qf, st, sc2, s_c, s_b, p, vf, va, plan);
        static_bodies<RB, RING, PH + 2>(lds, lo, full, qf, st, sc2, s_b, s_c, p, vf, va, plan);
    }
}

template <int RB, bool NT, bool KCOL>
__device__ __forceinline__ void run_blocks(RingStart<Ring<RB>::slots, NT, KCOL>& rs, char* lds, const bf16x8 (&qf)[RB][8],
                                           WaveState<RB>& st, float sc2, const int (&lim)[RB]) {
    constexpr int RING = Ring<RB>::slots;
    constexpr int NF = RING - 3;
    constexpr bool STATIC_RING = RB == 2 && KCOL;        // the wide tile
    if (rs.d0 == 0) return;
    RingPlan<RING>& plan = rs.plan;
    const LoadOffsetsT<NT, KCOL> full = rs.full;
    const int d0 = rs.d0;
    const int (&first)[NF + 1] = rs.first;
    const LaneOffsets lo = lane_offsets<KCOL>(rs.tid);
    // block 0 has landed when at most the NF younger blocks are in flight; loads of the caller
    // that are younger still (the query fragments) only make this wait longer
    f32x16 s_b[RB], s_c[RB];
    if (first[NF - 1] != 0) wait_blocks<NF>(); else wait_blocks<0>();
    ring_barrier();
    scores<RB, KCOL>(lds, lo, qf, s_b);

    // the plan of body 0, as the pieces would leave it
    plan.d_cur = d0;
    plan.d_nxt = first[0];
#pragma unroll
    for (int i = 0; i < NF; ++i) plan.fifo[i] = first[i + 1];
    plan.deep = NF >= 2 && plan.fifo[NF >= 2 ? NF - 2 : 0] != 0;
    plan.o_pv = (RING - 1) * SLOTB; plan.o_cur = 0; plan.o_nxt = SLOTB; plan.o_new = (RING - 2) * SLOTB;
    plan.piece(2);
    plan.piece(3);
    // body 0 has no block -1: its PV product runs on zero probabilities and block 0's (finite) values
    u32x4 p[RB][2], p2[RB][2];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) p[rb][0] = p[rb][1] = u32x4{0, 0, 0, 0};
    bf16x8 vf[8];
#pragma unroll
    for (int f = 0; f < 4; ++f) vf[f] = read_v_frag(lds, lo, f);
    VAddr va;                                                        // (body 0: block -1 is block 0's slot, see below)
#pragma unroll
    for (int db = 0; db < 4; ++db) va.a[db] = lds + lo.v[db];
    int pv_off = 0;
    for (;;) {
        // ---- fast stretch: bodies that need no descriptor, no mask and no table look-up
        const int n_fast = plan.fast_bodies();
        int n_left = n_fast;
        auto single = [&]() {
            wait_blocks<NF >= 2 ? NF - 1 : 0>();
            ring_barrier();
            const int next_pv_off = plan.o_cur;
            pipeline_body<RB, RING, true>(lds, pv_off, lo, full, qf, st, sc2, s_b, p, vf, va, plan, lim);
            pv_off = next_pv_off;
        };
        if constexpr (STATIC_RING) {
            // Long stretches (a query prefill's context split): groups of RING bodies with the ring slots
            // as compile-time constants (209-222 instead of 218-222 instructions per body; config-3 prefill
            // 0.503 -> 0.493 ms).  Bodies with run-time offsets first bring the ring round to slot 0: one
            // single body if that takes an odd number, then pairs.
            const FastSplit fs = split_fast<RING>(n_fast, plan.o_cur / SLOTB, pv_off == plan.o_cur);
            if (fs.supers > 0) {
                if (fs.pre & 1) single();
                for (int i = 0; i + 1 < fs.pre; i += 2) {
                    wait_blocks<NF - 1>(); ring_barrier();
                    int next_pv_off = plan.o_cur;
                    pipeline_body_pp<RB, RING>(lds, pv_off, lo, full, qf, st, sc2, s_b, s_c, p, vf, va, plan);
                    pv_off = next_pv_off;
                    wait_blocks<NF - 1>(); ring_barrier();
                    next_pv_off = plan.o_cur;
                    pipeline_body_pp<RB, RING>(lds, pv_off, lo, full, qf, st, sc2, s_c, s_b, p, vf, va, plan);
                    pv_off = next_pv_off;
                }
                for (int g = 0; g < fs.supers; ++g)
                    static_bodies<RB, RING, 0>(lds, lo, full, qf, st, sc2, s_b, s_c, p, vf, va, plan);
                n_left -= fs.pre + fs.supers * RING;
            }
        }
        for (int i = 0; i + 1 < n_left; i += 2) {                     // in pairs: the scores ping-pong between s_b and s_c
            wait_blocks<NF >= 2 ? NF - 1 : 0>();
            ring_barrier();
            int next_pv_off = plan.o_cur;
            // Narrow tile: the evenly spread body (+1.7 % measured).  Wide tile: its second set of
            // probability registers does not fit next to the 128 accumulators (the compiler parks 16
            // more values in the accumulation registers and copies them in and out, 18 instructions per
            // body), which eats the gain: it keeps the paired body.
            if constexpr (RB == 1) pipeline_body_even<RB, RING>(lds, pv_off, lo, full, qf, st, sc2, s_b, s_c, p, p2, vf, va, plan);
            else pipeline_body_pp<RB, RING>(lds, pv_off, lo, full, qf, st, sc2, s_b, s_c, p, vf, va, plan);
            pv_off = next_pv_off;
            wait_blocks<NF >= 2 ? NF - 1 : 0>();
            ring_barrier();
            next_pv_off = plan.o_cur;
            if constexpr (RB == 1) pipeline_body_even<RB, RING>(lds, pv_off, lo, full, qf, st, sc2, s_c, s_b, p2, p, vf, va, plan);
            else pipeline_body_pp<RB, RING>(lds, pv_off, lo, full, qf, st, sc2, s_c, s_b, p, vf, va, plan);
            pv_off = next_pv_off;
        }
        if (n_left & 1) single();
        if (n_fast > 0) plan.finish_fast(n_fast);
        // ---- generic body
        const int d_nxt = plan.d_nxt;
        if (d_nxt != 0) {
            // block j+1 must have landed: all but the NF-1 youngest blocks, when that many are in flight
            if (plan.deep) wait_blocks<NF >= 2 ? NF - 1 : 0>(); else wait_blocks<0>();
            // ... for every wavefront, all of which are then also done with block j-2's slot
            ring_barrier();
        }
        const int next_pv_off = plan.o_cur;
        pipeline_body<RB, RING, false>(lds, pv_off, lo, full, qf, st, sc2, s_b, p, vf, va, plan, lim);
        pv_off = next_pv_off;
        if (d_nxt == 0) break;
    }
    // the last block's PV product
#pragma unroll
    for (int f = 0; f < 8; ++f) {
        if (f >= 4) vf[f] = read_v_pv<RB == 1>(va, lds + pv_off, lo, f);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
            st.o[rb][f & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[f], __builtin_bit_cast(bf16x8, p[rb][f >> 2]),
                                                                      st.o[rb][f & 3], 0, 0, 0);
    }
}

// The block loop of a wavefront NONE of whose rows is a query row (a decode step fills 4 of a
// workgroup's 128 rows: one wavefront computes, the others only fetch).  Same control flow, same
// loads, waits and barriers as run_blocks, no matrix or vector work and no LDS reads.
template <int RB, bool NT, bool KCOL>
__device__ __forceinline__ void run_blocks_idle(RingStart<Ring<RB>::slots, NT, KCOL>& rs, char* lds) {
    constexpr int RING = Ring<RB>::slots;
    constexpr int NF = RING - 3;
    if (rs.d0 == 0) return;
    RingPlan<RING>& plan = rs.plan;
    const LoadOffsetsT<NT, KCOL> full = rs.full;
    if (rs.first[NF - 1] != 0) wait_blocks<NF>(); else wait_blocks<0>();
    ring_barrier();
    plan.d_cur = rs.d0;
    plan.d_nxt = rs.first[0];
#pragma unroll
    for (int i = 0; i < NF; ++i) plan.fifo[i] = rs.first[i + 1];
    plan.deep = NF >= 2 && plan.fifo[NF >= 2 ? NF - 2 : 0] != 0;
    plan.o_pv = (RING - 1) * SLOTB; plan.o_cur = 0; plan.o_nxt = SLOTB; plan.o_new = (RING - 2) * SLOTB;
    plan.piece(2);
    plan.piece(3);
    for (;;) {
        const int n_fast = plan.fast_bodies();
        for (int i = 0; i < n_fast; ++i) {
            wait_blocks<NF >= 2 ? NF - 1 : 0>();
            ring_barrier();
#pragma unroll
            for (int n = 0; n < LOADS_PER_BLOCK; ++n) issue_block_load(n, plan.new_k, plan.new_v, lds + plan.o_new, full);
            plan.fast_piece(0); plan.fast_piece(1); plan.fast_piece(2);
        }
        if (n_fast > 0) plan.finish_fast(n_fast);
        const int d_nxt = plan.d_nxt;
        if (d_nxt != 0) {
            if (plan.deep) wait_blocks<NF >= 2 ? NF - 1 : 0>(); else wait_blocks<0>();
            ring_barrier();
        }
        if (plan.d_new != 0)
            issue_block_loads(plan.new_k, plan.new_v, desc_n(plan.d_new), plan.ld.stride_b, lds + plan.o_new, full);
        if (d_nxt == 0) break;
        plan.piece(0); plan.piece(1); plan.piece(2); plan.piece(3);
    }
}

template <int RB>
__device__ __forceinline__ void init_state(WaveState<RB>& st) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        st.m[rb] = kUnset; st.l[rb] = 0.f;
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
// Query prefill: team = (split, KV head); grid = the context teams (padded to a multiple of 8) times
// n_qtiles, then the prefix+self teams likewise.
// Rows: R = qtile*BM + wave*32*RB + rb*32 + (lane & 31); query token = R / G, head = hk*G + R % G.
template <int RB, int G, bool NTL>
__global__ __launch_bounds__(NT) void flash_prefill_kernel(const QueryArgs a, int n_qtiles) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    constexpr int BM = NW * 32 * RB;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hi = lane >> 5;
    // Blocks of the context splits come first: they are the long ones, and the grid is planned so
    // that they fill the chip exactly once; the short prefix+self workgroups follow.
    int team, qtile, split, hk;
    const int ctx_teams = a.n_ctx_splits * a.n_kv_heads;
    const int ctx_blocks = (ctx_teams + 7) / 8 * 8 * n_qtiles;
    int bx = blockIdx.x, rq = blockIdx.y;                // position in the request's part of the grid; request
    if (NTL && a.n_req > 1) {
        // A batch on one tile per KV head (a decode step): the context workgroups of ALL requests
        // first, then every request's short prefix+self ones, in the order workgroups are dispatched
        // (x fastest, then y).  Dealt request by request, the short ones sit between the long ones
        // and leave their slots early, which spoils the balance when the long ones are few.
        const int short_blocks = (int)gridDim.x - ctx_blocks;
        const int lin = (int)blockIdx.y * (int)gridDim.x + (int)blockIdx.x;
        const int ctx_all = a.n_req * ctx_blocks;
        if (lin < ctx_all) { rq = lin / ctx_blocks; bx = lin - rq * ctx_blocks; }
        else { const int l2 = lin - ctx_all; rq = l2 / short_blocks; bx = ctx_blocks + (l2 - rq * short_blocks); }
    }
    if (bx < ctx_blocks) {
        team_of_block(bx, n_qtiles, team, qtile);
        if (team >= ctx_teams) return;
        // Under a tree plan the slots past the splits in use are empty and leave at once: with the
        // KV head as the fastest index they are the last workgroups of the context part instead of
        // sitting between the working ones (where they upset the even deal of one workgroup per CU:
        // 128K decode 99 us against 84 us for the same splits without empty slots in between).
        // One request on one tile per KV head (a decode step at batch 1: every workgroup resident at
        // once) reads faster in that order too, 87.4 against 89.8 us over 128K tokens -- the eight
        // heads of a token's 2 KB row are then fetched at about the same time; a batch does not
        // (config 5: 0.346 against 0.339 ms), its workgroups run in several rounds.
        if (a.split_ranges != nullptr || (n_qtiles == 1 && a.n_req == 1)) { hk = team % a.n_kv_heads; split = team / a.n_kv_heads; }
        else { split = team % a.n_ctx_splits; hk = team / a.n_ctx_splits; }
    } else {
        team_of_block(bx - ctx_blocks, n_qtiles, team, qtile);
        if (team >= a.n_kv_heads) return;
        split = a.n_ctx_splits; hk = team;
    }
    const KvView kv = load_view<QueryArgs>(rq);
    const int hq = a.n_q_heads, q_len = a.q_len;
    const long stride_b = (long)a.n_kv_heads * ROWB, head_b = (long)hk * ROWB;

    // the stream of K/V blocks; its first loads start before anything else
    const int causal_off = kv.self_len - q_len;
    const int R_lo = qtile * BM + wave * 32 * RB;
    const int tok_lo = min(R_lo / G, q_len - 1);
    const float inv_sqrt_d = 0.08838834764831845f;      // 1/sqrt(128)
    Stream walk;
    float sc2 = inv_sqrt_d * LOG2E;
    int vis_lo = 0;
    if (split < a.n_ctx_splits) {
        long t0, t1;
        ctx_split_range(a, kv, split, t0, t1);
        // An empty split (a slot past the splits a tree plan uses; in a batch, a split past the end
        // of a request's context) is one the merge never looks at: the whole workgroup leaves
        // here, before any barrier or load.
        if (t0 >= t1) return;
        walk.init_ctx(kv.cu, kv.k_chunks, kv.v_chunks, kv.n_chunks, (int)t0, (int)t1, stride_b, head_b);
        sc2 = inv_sqrt_d / kv.temperature * LOG2E;
    } else {
        // rows of this workgroup see the causal segment up to the last valid row's limit
        const int wg_tok_hi = min((qtile * BM + BM - 1) / G, q_len - 1);
        walk.init_seq((const char*)kv.k_prefix + head_b, (const char*)kv.v_prefix + head_b, kv.prefix_len,
                      (const char*)kv.k_self + head_b, (const char*)kv.v_self + head_b, wg_tok_hi + causal_off + 1, stride_b);
        vis_lo = tok_lo + causal_off;
    }
    // the wide tile reads K from the column-major form (measured: wide prefill 0.524 -> 0.513 ms; the narrow
    // tile, bound by its LDS and load traffic rather than by instruction issue, loses 1 % with it)
    RingStart<Ring<RB>::slots, NTL, RB == 2 && !NTL> rs;
    start_stream(rs, walk, lds, __builtin_amdgcn_readfirstlane(vis_lo), tid);

    // Q fragments (B operand: row = lane & 31, dims 16*ks + 8*hi .. +7)
    bf16x8 qf[RB][8];
    int lim[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int R = qtile * BM + wave * 32 * RB + rb * 32 + l32;
        const int tok = R / G, g = R % G;
        const bool valid = tok < q_len;
        lim[rb] = (valid ? tok : q_len - 1) + causal_off;
        const char* qp = (const char*)a.q + (((long)rq * q_len + tok) * hq + hk * G + g) * ROWB + hi * 16;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            u32x4 w = {0, 0, 0, 0};
            if (valid) w = *(const u32x4*)(qp + ks * 32);
            qf[rb][ks] = __builtin_bit_cast(bf16x8, w);
        }
    }

    WaveState<RB> st;
    init_state<RB>(st);
    // a wavefront without a single query row (R_lo is its first row) only fetches
    if (RB == 1 && __builtin_amdgcn_readfirstlane(R_lo / G) >= q_len) run_blocks_idle<RB>(rs, lds);
    else run_blocks<RB>(rs, lds, qf, st, sc2, lim);

    // ---- block result (Appendix C.1): normalised values + natural-log LogSumExp
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int R = qtile * BM + wave * 32 * RB + rb * 32 + l32;
        const int tok = R / G, g = R % G;
        const float lt = st.l[rb] + __shfl_xor(st.l[rb], 32);
        if (tok >= q_len) continue;
        const float inv = lt > 0.f ? 1.f / lt : 0.f;
        const long unit = ((long)(a.req_base + rq) * q_len + tok) * hq + hk * G + g;
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
// heaviest (last) tile first.  Writes the final bf16 output.  `vblock` is the tile's index in the
// order team_of_block() defines (the blockIdx of a launch with one workgroup per tile).
template <int RB, int G>
__device__ __forceinline__ void encode_tile(const EncodeArgs a, const int n_qtiles, const int vblock, char* const lds, const int tid) {
    constexpr int BM = NW * 32 * RB;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hi = lane >> 5;
    // Narrow tile: a wavefront outside its block loop (set-up, first loads, output) goes ahead of the wavefronts
    // of the CU's other workgroup that are inside theirs, so that the CU spends more of its time with both
    // workgroups in their loops (512 chunks of 256 tokens: 0.773 -> 0.764 ms; 2048-token chunks unchanged).
    if constexpr (RB == 1) __builtin_amdgcn_s_setprio(3);
    int team, member;
    team_of_block(vblock, n_qtiles, team, member);
    if (team >= a.n_chunks * a.n_kv_heads) return;
    const int qtile = n_qtiles - 1 - member;
    const int chunk = team / a.n_kv_heads, hk = team % a.n_kv_heads;
    // (chunks of one length: no table read in front of the tile's first loads)
    const int c0 = a.uniform_chunks ? chunk * a.max_chunk_len : a.cu ? a.cu[chunk] : 0;
    const int len = a.uniform_chunks ? a.max_chunk_len : a.cu ? a.cu[chunk + 1] - c0 : a.total_rows;
    if ((long)qtile * BM >= (long)len * G) return;
    const int hq = a.n_q_heads;
    const long stride_b = (long)a.n_kv_heads * ROWB, head_b = (long)hk * ROWB;

    // the stream of K/V blocks (prefix, then the chunk up to this tile's last row); its first loads
    // start before anything else
    const int R_lo = qtile * BM + wave * 32 * RB;
    const int tok_lo = min(R_lo / G, len - 1);
    const int wg_tok_hi = min((qtile * BM + BM - 1) / G, len - 1);
    Stream walk;
    walk.init_seq((const char*)a.k_prefix + head_b, (const char*)a.v_prefix + head_b, a.prefix_len,
              (const char*)a.k + (long)c0 * stride_b + head_b, (const char*)a.v + (long)c0 * stride_b + head_b,
              wg_tok_hi + 1, stride_b);
    RingStart<Ring<RB>::slots, false, RB == 2> rs;
    start_stream(rs, walk, lds, __builtin_amdgcn_readfirstlane(tok_lo), tid);

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

    WaveState<RB> st;
    init_state<RB>(st);
    if constexpr (RB == 1) __builtin_amdgcn_s_setprio(0);
    run_blocks<RB>(rs, lds, qf, st, 0.08838834764831845f * LOG2E, lim);
    if constexpr (RB == 1) __builtin_amdgcn_s_setprio(3);

    if constexpr (RB == 2) {
        // Wide tile (chunks beyond 4096 tokens: long streams, the output is a small part of a tile's
        // time): every lane stores its 4-dim pieces directly.  (Staging through LDS as below makes the
        // compiler park a hundred more values in the accumulation registers of this kernel.)
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
    } else {
        // ---- output: the wavefront's rows go through LDS (the ring is idle now) so that they leave as
        // whole 256-byte rows, 16 bytes per lane: the G heads of a token are neighbours in memory, and a
        // store instruction then writes up to 1 KB of consecutive bytes instead of 64 scattered pieces.
        ring_barrier();                                        // every wavefront is done with the last block's slot
        char* stage = lds + (long)wave * (RB * 32 * ROWB);     // RB * 8 KB of this wavefront's own
    #pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const int R = qtile * BM + wave * 32 * RB + rb * 32 + l32;
            const int tok = R / G, g = R % G;
            const float lt = st.l[rb] + __shfl_xor(st.l[rb], 32);
            const float inv = tok < len ? 1.f / lt : 0.f;      // a valid row always sees itself
            char* row = stage + (rb * 32 + l32) * ROWB;
    #pragma unroll
            for (int db = 0; db < 4; ++db)
    #pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    bf16x4 w;
    #pragma unroll
                    for (int e = 0; e < 4; ++e) w[e] = (__bf16)(st.o[rb][db][4 * q4 + e] * inv);
                    // 16-byte chunk 4*db + q4 of the row, XOR-swizzled by the row; this lane's half of it
                    *(bf16x4*)(row + (((4 * db + q4) ^ (l32 & 15)) << 4) + 8 * hi) = w;
                }
            if (a.lse && hi == 0 && tok < len) a.lse[(long)(hk * G + g) * a.total_rows + c0 + tok] = (st.m[rb] + __builtin_amdgcn_logf(lt)) * LN2;
        }
        // (the staging area is the wavefront's own: no barrier, the LDS operations of one wavefront complete in order)
        {
            const int c16 = lane & 15, r4 = lane >> 4;
    #pragma unroll
            for (int i = 0; i < RB * 8; ++i) {
                const int lr = 4 * i + r4;                     // row of the wavefront's RB * 32
                const int R = qtile * BM + wave * 32 * RB + lr;
                const int tok = R / G, g = R % G;
                const u32x4 w = *(const u32x4*)(stage + lr * ROWB + ((c16 ^ (lr & 15)) << 4));
                if (tok < len) *(u32x4*)((char*)a.out + ((long)(c0 + tok) * hq + hk * G + g) * ROWB + c16 * 16) = w;
            }
        }
    }
}

// Two launch shapes.  One workgroup per tile (rounds == 0): the hardware hands out the tiles.
// Resident workgroups (rounds > 0; the grid is 8 * slots_per_xcd workgroups, as many as the chip holds
// at once): each walks `rounds` tiles of its own XCD's list, so the ~3 us between the end of one
// workgroup and the start of the next on the same CU are paid once, not per tile.  A tile's weight
// falls with its index inside a team (the last query tile of a chunk sees the most keys), so the
// direction of the walk alternates from round to round: the workgroup that drew the heaviest tile
// of a round draws the lightest of the next.  Used when all chunks have the same length, where this
// static deal is balanced.
template <int RB, int G>
__global__ __launch_bounds__(NT) void flash_encode_kernel(const EncodeArgs a, int n_qtiles, int slots_per_xcd, int rounds) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    if constexpr (RB == 2) {
        // (the wide tile always runs one tile per workgroup: its chunks are long, and a tile loop around
        // its block loop costs it registers it does not have)
        encode_tile<RB, G>(a, n_qtiles, blockIdx.x, lds, threadIdx.x);
    } else {
        if (rounds == 0) { encode_tile<RB, G>(a, n_qtiles, blockIdx.x, lds, threadIdx.x); return; }
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        for (int k = 0; k < rounds; ++k) {
            // (every wavefront has read its output rows back from LDS before the next tile's loads overwrite them)
            if (k > 0) ring_barrier();
            const int v = k * slots_per_xcd + ((k & 1) ? slots_per_xcd - 1 - slot : slot);
            encode_tile<RB, G>(a, n_qtiles, v * 8 + xcd, lds, tile_thread_index());
        }
    }
}

template <int RB, int G, bool NTL>
hipError_t launch_prefill_t(const QueryArgs& a, dim3 grid, int n_qtiles, hipStream_t s) {
    hipError_t e = hipFuncSetAttribute((const void*)flash_prefill_kernel<RB, G, NTL>, hipFuncAttributeMaxDynamicSharedMemorySize, Ring<RB>::slots * SLOTB);
    if (e != hipSuccess) return e;
    flash_prefill_kernel<RB, G, NTL><<<grid, NT, Ring<RB>::slots * SLOTB, s>>>(a, n_qtiles);
    return hipGetLastError();
}

template <int RB, int G>
hipError_t launch_encode_t(const EncodeArgs& a, unsigned grid, int n_qtiles, int slots_per_xcd, int rounds, hipStream_t s) {
    hipError_t e = hipFuncSetAttribute((const void*)flash_encode_kernel<RB, G>, hipFuncAttributeMaxDynamicSharedMemorySize, Ring<RB>::slots * SLOTB);
    if (e != hipSuccess) return e;
    flash_encode_kernel<RB, G><<<grid, NT, Ring<RB>::slots * SLOTB, s>>>(a, n_qtiles, slots_per_xcd, rounds);
    return hipGetLastError();
}

template <int RB, bool NTL>
hipError_t launch_prefill_g(int group, const QueryArgs& a, dim3 grid, int n_qtiles, hipStream_t s) {
    switch (group) {
        case 1: return launch_prefill_t<RB, 1, NTL>(a, grid, n_qtiles, s);
        case 2: return launch_prefill_t<RB, 2, NTL>(a, grid, n_qtiles, s);
        case 4: return launch_prefill_t<RB, 4, NTL>(a, grid, n_qtiles, s);
        default: return launch_prefill_t<RB, 8, NTL>(a, grid, n_qtiles, s);
    }
}

template <int RB>
hipError_t launch_encode_g(int group, const EncodeArgs& a, unsigned grid, int n_qtiles, int slots_per_xcd, int rounds, hipStream_t s) {
    switch (group) {
        case 1: return launch_encode_t<RB, 1>(a, grid, n_qtiles, slots_per_xcd, rounds, s);
        case 2: return launch_encode_t<RB, 2>(a, grid, n_qtiles, slots_per_xcd, rounds, s);
        case 4: return launch_encode_t<RB, 4>(a, grid, n_qtiles, slots_per_xcd, rounds, s);
        default: return launch_encode_t<RB, 8>(a, grid, n_qtiles, slots_per_xcd, rounds, s);
    }
}

}  // namespace

int flash_block_rows(int rows_per_kv_head) { return rows_per_kv_head > 128 ? 256 : 128; }

// Query prefill: over a short context a workgroup's stream is a few dozen blocks, and what it spends
// around them (descriptor and table reads, first loads, the partial results it writes and the merge
// reads back) weighs as much as the blocks; the narrow tile then wins because two of its workgroups
// share a CU and because half as many splits reach the same number of workgroups.  Measured with 256
// query rows (64 tokens x 4 heads per KV head give the same picture): 2.5K context 0.047 against
// 0.064 ms, 10K 0.078 / 0.089, 16K 0.102 / 0.113, 32K 0.160 / 0.168, 48K 0.229 / 0.232, 64K equal, 128K
// 0.537 / 0.527.  Up to 12K tokens one narrow workgroup per CU is enough, beyond that two.
// With more query rows there are more row tiles per KV head, fewer splits and longer streams, and the
// wide tile's better steady state wins sooner (narrow / wide, ms): 512 tokens x 4 heads over 24K and 32K
// equal; 1024 x 4 over 16K 0.295 / 0.300, 24K 0.422 / 0.415, 32K 0.539 / 0.526, 40K 0.638 / 0.614;
// 2048 x 4 over 8K 0.341 / 0.335, 16K 0.572 / 0.551, 24K 0.806 / 0.767, 32K 1.037 / 0.977.
long flash_prefill_narrow_tile_max_ctx(int rows_per_kv_head) {
    return rows_per_kv_head >= 8192 ? 6144 : rows_per_kv_head >= 4096 ? 20480 : 40960;
}
int flash_prefill_block_rows(int rows_per_kv_head, long max_ctx) {
    if (max_ctx <= flash_prefill_narrow_tile_max_ctx(rows_per_kv_head)) return 128;
    return flash_block_rows(rows_per_kv_head);
}
int flash_prefill_target_workgroups(int rows_per_kv_head, long max_ctx) {
    return max_ctx > kPrefillOneWorkgroupPerCuMaxCtx && max_ctx <= flash_prefill_narrow_tile_max_ctx(rows_per_kv_head) ? 512 : 256;
}

hipError_t launch_flash_prefill(const QueryArgs& a, int block_rows, hipStream_t s) {
    const int group = a.n_q_heads / a.n_kv_heads;
    const int rows = a.q_len * group;
    const int bm = block_rows == 256 ? 256 : 128;
    const int n_qtiles = (rows + bm - 1) / bm;
    const int ctx_teams = a.n_ctx_splits * a.n_kv_heads;
    // x is a multiple of 8, so the workgroups of every request start on the same XCD phase
    const dim3 grid((unsigned)(((ctx_teams + 7) / 8 * 8 + (a.n_kv_heads + 7) / 8 * 8) * n_qtiles), (unsigned)a.n_req);
    if (bm == 256) return launch_prefill_g<2, false>(group, a, grid, n_qtiles, s);
    // one row tile: every K/V block is fetched by one workgroup and never again -> non-temporal loads
    return n_qtiles == 1 ? launch_prefill_g<1, true>(group, a, grid, n_qtiles, s) : launch_prefill_g<1, false>(group, a, grid, n_qtiles, s);
}

hipError_t launch_flash_encode(const EncodeArgs& a, hipStream_t s) {
    if (a.total_rows == 0) return hipSuccess;
    const int group = a.n_q_heads / a.n_kv_heads;
    const int rows = a.max_chunk_len * group;
    // The encode of a chunk is many short streams (a query tile sees only the keys before it), so
    // the per-workgroup start-up and wind-down weigh more than in the prefill: up to 4K-token chunks
    // the narrow tile wins, because two of its workgroups share a CU and cover for each other
    // (measured: +4..7 % at 2048-token chunks, +15..29 % at 256..512, -1.5 % at 8192).
    const int bm = a.max_chunk_len > 4096 ? flash_block_rows(rows) : 128;
    const int n_qtiles = (rows + bm - 1) / bm;
    const int teams = a.n_chunks * a.n_kv_heads;
    unsigned grid = (unsigned)((teams + 7) / 8 * 8 * n_qtiles);
    // Resident workgroups (two of the narrow tile per CU, walking the tiles in a fixed deal) for many
    // short chunks of one length: there a tile is a handful of blocks and the ~3 us between two
    // workgroups on a CU weigh most (measured: 512 x 256 tokens 0.821 -> 0.798 ms, 20 x 512 0.087 ->
    // 0.084 ms).  Longer chunks are better off with the hardware handing out the tiles: CUs differ in
    // speed by a few per cent and a fixed deal ends with the slowest (64 x 2048: 2.34 -> 2.41 ms).
    int slots_per_xcd = 0, rounds = 0;
    if (a.uniform_chunks && bm == 128 && a.max_chunk_len <= 1024) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus >= 8) {
            const int resident = cus / 8 * 2;                                // per XCD
            const int per_xcd = (int)(grid / 8);
            if (per_xcd >= 4 * resident) {
                slots_per_xcd = resident;
                rounds = (per_xcd + resident - 1) / resident;
                grid = (unsigned)(8 * resident);
            }
        }
    }
    return bm == 256 ? launch_encode_g<2>(group, a, grid, n_qtiles, slots_per_xcd, rounds, s)
                     : launch_encode_g<1>(group, a, grid, n_qtiles, slots_per_xcd, rounds, s);
}

}  // namespace ape
