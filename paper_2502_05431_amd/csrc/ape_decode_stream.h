// Scalar bookkeeping of the decode kernel: which tokens a wavefront streams and where their K/V
// rows are.  Wavefront-uniform integer and pointer arithmetic with no GPU instruction in it, so the
// same code compiles for the host, where a simulation drives it through ragged chunk tables, splits
// that start and end inside chunks, empty splits and tables shorter than the stated context, and
// checks what the kernel relies on: every token of a split is delivered once, in order, as tiles of
// 1..32 rows that stay inside one chunk and inside that chunk's rows.
//
// The includer defines APE_STREAM_FN (function qualifiers), the two table readers
// ape_stream_load_i32 / ape_stream_load_ptr (scalar loads on the GPU, plain reads on the host),
// ape_stream_find_chunk(cu, n_chunks, t) = the largest c with cu[c] <= t, and the view type: any
// struct with the fields cu, k_chunks, v_chunks, n_chunks.
#pragma once
#include <stdint.h>

namespace ape {

constexpr int kDecodeWaves = 4;                // wavefronts of a decode workgroup
constexpr int kDecodeTile = 32;                // tokens per wavefront tile

// Wavefront `wave`'s share [lo, hi) of the split [t0, t1): contiguous, a multiple of the tile except
// at the end; empty for an empty split.
APE_STREAM_FN void decode_wave_share(long t0, long t1, int wave, long& lo, long& hi) {
    const long per = t0 < t1 ? ((t1 - t0 + kDecodeWaves - 1) / kDecodeWaves + kDecodeTile - 1) / kDecodeTile * kDecodeTile : 0;
    lo = t0 + wave * per;
    hi = t1 < lo + per ? t1 : lo + per;
}

// Shares of the prefix (np rows) and of the query's own KV (ns rows): the prefix is dealt from
// wavefront 0 upwards and the own KV from the last wavefront down, so a short prefix and a short
// own span land on different wavefronts.
APE_STREAM_FN void decode_plain_shares(int np, int ns, int wave, int& pb, int& pe, int& sb, int& se) {
    const int perp = ((np + kDecodeWaves - 1) / kDecodeWaves + kDecodeTile - 1) / kDecodeTile * kDecodeTile;
    const int pers = ((ns + kDecodeWaves - 1) / kDecodeWaves + kDecodeTile - 1) / kDecodeTile * kDecodeTile;
    pb = np < wave * perp ? np : wave * perp;
    pe = np < pb + perp ? np : pb + perp;
    sb = ns < (kDecodeWaves - 1 - wave) * pers ? ns : (kDecodeWaves - 1 - wave) * pers;
    se = ns < sb + pers ? ns : sb + pers;
}

// One wavefront's token stream: up to two plain segments, or a range of the pooled contexts
// walked through the chunk table.  next() yields tiles of <= 32 tokens that never straddle a
// segment or chunk end.
struct DecodeStream {
    const int32_t* cu;                 // non-NULL: context range [t, te) through the chunk table (scalar loads)
    const void* const* k_chunks;
    const void* const* v_chunks;
    int n_chunks;
    int t, te, c0, c1;
    int c, c_loaded;                   // c_loaded: the chunk whose base pointers kc, vc hold (-1: none)
    const char *kc, *vc;
    const char *k0, *v0, *k1, *v1;    // plain segments
    int n0, n1;
    int seg, j;
    long stride_b, head_b;

    template <typename View>
    APE_STREAM_FN void init_ctx(const View& kv, long t_, long te_, long stride_b_, long head_b_) {
        cu = kv.cu; k_chunks = kv.k_chunks; v_chunks = kv.v_chunks; n_chunks = kv.n_chunks;
        t = (int)t_; te = (int)te_; stride_b = stride_b_; head_b = head_b_; c = 0; c0 = 0; c1 = 0;
        seg = 2; j = 0; n0 = n1 = 0; k0 = v0 = k1 = v1 = nullptr;
        c_loaded = -1; kc = vc = nullptr;
        if (t < te) {
            c = ape_stream_find_chunk(cu, n_chunks, t);                // the largest c with cu[c] <= t
            c0 = ape_stream_load_i32(cu + c); c1 = ape_stream_load_i32(cu + c + 1);
        } else {
            te = t;
        }
    }
    APE_STREAM_FN void init_plain(const char* k0_, const char* v0_, int n0_, const char* k1_, const char* v1_, int n1_, long stride_b_) {
        cu = nullptr; k_chunks = v_chunks = nullptr; n_chunks = 0; c = 0; c0 = c1 = 0;
        t = te = 0; stride_b = stride_b_; head_b = 0;
        k0 = k0_; v0 = v0_; n0 = n0_; k1 = k1_; v1 = v1_; n1 = n1_;
        seg = 0; j = 0; c_loaded = -1; kc = vc = nullptr;
    }
    APE_STREAM_FN bool next(const char*& kb, const char*& vb, int& nv) {
        if (cu) {
            if (t >= te) return false;
            while (t >= c1) {
                if (c + 1 >= n_chunks) { t = te; return false; }   // table shorter than total_ctx: stay in bounds
                ++c; c0 = c1; c1 = ape_stream_load_i32(cu + c + 1);
            }
            const int e = c1 < te ? c1 : te;
            nv = e - t < kDecodeTile ? e - t : kDecodeTile;
            if (c != c_loaded) {                                    // the table is read once per chunk, not per tile
                kc = (const char*)ape_stream_load_ptr(k_chunks + c) + head_b;
                vc = (const char*)ape_stream_load_ptr(v_chunks + c) + head_b;
                c_loaded = c;
            }
            kb = kc + (long)(t - c0) * stride_b;
            vb = vc + (long)(t - c0) * stride_b;
            t += nv;
            return true;
        }
        if (seg == 0 && j >= n0) { seg = 1; j = 0; }
        if (seg == 1 && j >= n1) seg = 2;
        if (seg >= 2) return false;
        const int n = seg == 0 ? n0 : n1;
        nv = n - j < kDecodeTile ? n - j : kDecodeTile;
        kb = (seg == 0 ? k0 : k1) + (long)j * stride_b;
        vb = (seg == 0 ? v0 : v1) + (long)j * stride_b;
        j += nv;
        return true;
    }
};

}  // namespace ape
