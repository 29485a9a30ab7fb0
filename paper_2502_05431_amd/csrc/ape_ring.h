// Scalar bookkeeping of the flash kernels: the stream of K/V blocks of one workgroup and the ring
// of LDS slots they pass through.  Everything here is wavefront-uniform integer and pointer
// arithmetic with no GPU instruction in it, so the same code compiles for the host: the CPU tests
// drive it through every kind of stream (segment ends, partial blocks, the causal diagonal,
// stretches of full blocks) and check what the kernels rely on -- every block is loaded once, in
// bounds, into a free slot; every body finds its three blocks where it looks for them; a fast
// body never meets a block that needs a mask.
//
// The includer defines APE_RING_FN (function qualifiers), the table readers ape_ring_load_i32 /
// ape_ring_load_ptr / ape_ring_load_chunk (scalar loads on the GPU, plain reads on the host) and
// ape_ring_find_chunk(cu, n_chunks, t) = the largest c with cu[c] <= t (a search across the lanes
// on the GPU, a plain one on the host).
#pragma once
#include <stdint.h>

namespace ape {

constexpr int BLK = 32;                      // KV tokens per block
constexpr int ROWB = 128 * 2;                // bytes of one head's K or V row (head_dim 128, bf16)
constexpr int KVB = BLK * ROWB;              // 8 KB: one block of K (or V) rows
constexpr int SLOTB = 2 * KVB;               // one ring slot: K rows then V rows

// A block = n_valid (1..32) consecutive tokens of one segment, described to the compute side by
// one integer: n_valid | (j0 + 1) << 6, j0 = index of row 0 inside its causal segment or -1 (no
// causal mask).  0 = no block.
APE_RING_FN int desc_n(int d) { return d & 63; }
APE_RING_FN int desc_j0(int d) { return (d >> 6) - 1; }

// The K/V rows of one workgroup as a stream of blocks: a list of segments (runs of rows at a fixed
// stride), each cut into blocks of 32 rows.  Two segment sources share the type (and therefore
// one instantiation of the pipeline): a range [t, t1) of the pooled contexts, cut at chunk ends
// through the chunk table (no mask), or a plain segment (the prefix) followed by a causal one
// (self KV / own chunk).  Everything here is wavefront-uniform and lives in scalar registers;
// the per-block path is a handful of scalar instructions, the tables are read (with scalar
// loads) only when a segment ends.
struct Stream {
    const char *k, *v;               // row 0 of the next block (this KV head)
    int rem;                         // rows left in the current segment; 0 = stream exhausted
    int run;                         // full blocks handed out back to back from the current segment
    int j0, jstep;                   // causal index of that row (-1: none) and its step per block
    long stride_b, head_b;
    // context source (cu != NULL)
    const int32_t* cu;
    const void* const* k_chunks;
    const void* const* v_chunks;
    int n_chunks, c, c0, c1, t, t1;  // chunk c = [c0, c1) holds pooled index t, the next undelivered row
    // sequence source: the causal segment still to come (nc == 0: none)
    const char *kc, *vc;
    int nc;

    // Opens the segment that starts at pooled index t (t < t1).
    APE_RING_FN void open_ctx() {
        const void *kb = nullptr, *vb = nullptr;
        bool have = false;
        while (t >= c1) {                                          // the next chunk, skipping empty ones
            if (c + 1 >= n_chunks) return;                         // table shorter than total_ctx: stop, stay in bounds
            ++c; c0 = c1;
            ape_ring_load_chunk(cu + c + 1, k_chunks + c, v_chunks + c, c1, kb, vb);   // one round trip per chunk
            have = true;
        }
        if (!have) { kb = ape_ring_load_ptr(k_chunks + c); vb = ape_ring_load_ptr(v_chunks + c); }
        const long off = (long)(t - c0) * stride_b + head_b;
        k = (const char*)kb + off;
        v = (const char*)vb + off;
        const int e = c1 < t1 ? c1 : t1;
        rem = e - t; t = e;
    }
    APE_RING_FN void init_ctx(const int32_t* cu_, const void* const* k_chunks_, const void* const* v_chunks_, int n_chunks_,
                              int t0_, int t1_, long stride_b_, long head_b_) {
        cu = cu_; k_chunks = k_chunks_; v_chunks = v_chunks_; n_chunks = n_chunks_;
        stride_b = stride_b_; head_b = head_b_;
        k = v = kc = vc = nullptr; nc = 0; rem = 0; run = 0; j0 = -1; jstep = 0;
        t = t0_; t1 = t1_; c = 0; c0 = c1 = 0;
        if (t < t1 && cu != nullptr && n_chunks > 0) {
            c = ape_ring_find_chunk(cu, n_chunks, t);              // the largest c with cu[c] <= t
            c0 = ape_ring_load_i32(cu + c); c1 = ape_ring_load_i32(cu + c + 1);
            open_ctx();
        }
    }
    APE_RING_FN void init_seq(const char* kp, const char* vp, int np, const char* kc_, const char* vc_, int nc_, long stride_b_) {
        cu = nullptr; k_chunks = v_chunks = nullptr; n_chunks = c = c0 = c1 = t = t1 = 0; head_b = 0;
        stride_b = stride_b_;
        kc = kc_; vc = vc_; nc = nc_;
        k = kp; v = vp; rem = np; run = 0; j0 = -1; jstep = 0;
        if (rem == 0) next_segment();
    }
    APE_RING_FN void next_segment() {
        const int run_before = run;
        run = 0;
        if (cu != nullptr) {
            if (t < t1) {
                // A context that starts exactly where the rows handed out so far end (a packed cache, or
                // neighbouring pages) continues the run of full blocks: same stride, no causal index, so
                // the blocks on either side of the boundary are indistinguishable to the compute side.
                // (After a partial block run_before is 0 already.)
                const char *k_end = k, *v_end = v;
                open_ctx();
                if (rem > 0 && k == k_end && v == v_end) run = run_before;
            }
        } else if (nc > 0) {
            k = kc; v = vc; rem = nc; nc = 0; j0 = 0; jstep = BLK;
        }
    }
    // Hands out the next block (rem > 0) and steps past it.
    APE_RING_FN int take(const char*& bk, const char*& bv) {
        const int n = rem < BLK ? rem : BLK;
        const int d = n | ((j0 + 1) << 6);
        bk = k; bv = v;
        k += BLK * stride_b; v += BLK * stride_b;
        rem -= n; j0 += jstep;
        run = n == BLK ? run + 1 : 0;
        if (__builtin_expect(rem == 0, 0)) next_segment();
        return d;
    }
};

// Scalar bookkeeping of the ring, advanced once per loop body.  A wavefront issues one
// instruction every few cycles whatever its kind, so this bookkeeping is cut into small pieces
// that the pipeline places between the MFMAs of the PV product, where issue slots are free.
// At the top of body j:
//   - blocks j-1, j, j+1 are resident (PV of j-1, softmax of j, K Q^T of j+1 run in this body),
//     blocks j+2 .. j+RING-3 are in flight, and the loads of block j+RING-2 start, into the slot
//     block j-2 has left;
//   - d_cur / d_nxt describe blocks j and j+1, fifo[q] block j+2+q (0 = no such block), the last
//     entry being the block whose loads start now (d_new, new_k, new_v);
//   - o_pv / o_cur / o_nxt / o_new are the ring offsets of blocks j-1, j, j+1 and of the new block.
template <int RING>
struct RingPlan {
    static constexpr int NF = RING - 3;
    Stream ld;
    int fifo[NF];
    int d_cur, d_nxt, d_new;
    const char *new_k, *new_v;
    int o_pv, o_cur, o_nxt, o_new;
    bool deep;                      // NF-1 blocks younger than j+1 are in flight (else: wait for all)
    bool cur_masked;
    int vis_lo;

    APE_RING_FN bool masked(int d) const {
        return desc_n(d) < BLK || (desc_j0(d) >= 0 && desc_j0(d) + BLK - 1 > vis_lo);
    }
    // The pieces, in order, of "advance to the next body" (piece indices beyond the last do nothing).
    APE_RING_FN void piece(int i) {
        if (i == 0) {                                  // the descriptors move up
            d_cur = d_nxt;
            d_nxt = fifo[0];
#pragma unroll
            for (int q = 0; q + 1 < NF; ++q) fifo[q] = fifo[q + 1];
            fifo[NF - 1] = 0;
            deep = NF >= 2 && fifo[NF >= 2 ? NF - 2 : 0] != 0;
        } else if (i == 1) {                           // the ring turns
            o_new = o_pv; o_pv = o_cur; o_cur = o_nxt;
            o_nxt = o_nxt + SLOTB == RING * SLOTB ? 0 : o_nxt + SLOTB;
        } else if (i == 2) {                           // the block whose loads start next
            d_new = 0;
            if (d_nxt != 0 && ld.rem > 0) { d_new = ld.take(new_k, new_v); fifo[NF - 1] = d_new; }
        } else if (i == 3) {
            cur_masked = masked(d_cur);
        }
    }
    // The same advance inside a fast stretch (see run_blocks): every block is a full block of the
    // loader's current segment, so only the pointers and the ring offsets move.
    APE_RING_FN void fast_piece(int i) {
        if (i == 0) {
            new_k = ld.k; new_v = ld.v;
        } else if (i == 1) {
            ld.k += BLK * ld.stride_b; ld.v += BLK * ld.stride_b;
        } else if (i == 2) {
            o_new = o_pv; o_pv = o_cur; o_cur = o_nxt;
            o_nxt = o_nxt + SLOTB == RING * SLOTB ? 0 : o_nxt + SLOTB;
        }
    }
    // Number of bodies of a fast stretch that may start now (0: none).  In a stretch every block
    // described here (j .. j+RING-2) and every block taken is a full block of the loader's current
    // segment, handed out back to back, and the blocks whose softmax runs need no mask; so the
    // bodies need no descriptor, no branch and no table look-up, and finish_fast() can rebuild
    // the descriptors from the loader's position.
    APE_RING_FN int fast_bodies() const {
        if (ld.run < RING - 1) return 0;
        int n = ld.rem / BLK;
        if (ld.jstep != 0) { const int clear = (vis_lo - desc_j0(d_cur) + 1) / BLK; n = n < clear ? n : clear; }
        return n > 0 ? n : 0;
    }
    APE_RING_FN void finish_fast(int n) {
        ld.rem -= n * BLK;
        ld.j0 += n * ld.jstep;
        ld.run += n;
        // the RING-1 blocks described are the last RING-1 taken; the newest is the prepared one
        auto d_age = [&](int a) { return BLK | ((ld.jstep != 0 ? ld.j0 - BLK * (a + 1) + 1 : 0) << 6); };
        d_new = d_age(0);
#pragma unroll
        for (int q = 0; q < NF; ++q) fifo[NF - 1 - q] = d_age(q);
        d_nxt = d_age(NF);
        d_cur = d_age(NF + 1);
        deep = NF >= 2;
        cur_masked = masked(d_cur);
        if (ld.rem == 0) ld.next_segment();
    }
};

// How a fast stretch of n bodies is run when block j of its first body sits in ring slot `phase`:
// `pre` bodies with run-time slot offsets bring the ring round to slot 0, then `supers` groups of RING
// bodies run with compile-time slots, the rest again with run-time offsets.  For long stretches only
// (the groups are a second copy of the loop body, RING times over).
struct FastSplit { int pre, supers; };
// `first`: the stretch starts with the stream's very first body, whose "block j-1" is block 0's own
// slot and not the slot before it in the ring: that body must run with run-time offsets.
template <int RING>
APE_RING_FN FastSplit split_fast(int n, int phase, bool first) {
    FastSplit f{0, 0};
    if (n < 4 * RING) return f;
    f.pre = phase == 0 && !first ? 0 : RING - phase;
    f.supers = (n - f.pre) / RING;
    return f;
}

}  // namespace ape
