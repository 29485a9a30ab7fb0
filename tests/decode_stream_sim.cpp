// Host simulation of the scalar bookkeeping of the decode kernel (csrc/ape_decode_stream.h): the
// header is compiled for the host and driven through ragged chunk tables (empty chunks, chunks of
// one row, chunks longer than several tiles), every split length the planner can choose, explicit
// split ranges as the tree entry point passes them, tables that hold fewer tokens than the stated
// context, and every prefix / own-KV length up to several tiles.  Checked: each tile has 1..32 rows,
// lies inside one chunk and inside that chunk's rows, K and V addresses agree, tiles of a wavefront
// come in order without gaps, and the four wavefronts of all splits together deliver every token
// exactly once.
// Build: g++ -O1 -std=c++17 [-fsanitize=address,undefined] decode_stream_sim.cpp; exit status 0 = all cases pass.
#include <cstdint>
#include <cstdio>
#include <random>
#include <vector>

#define APE_STREAM_FN inline
static inline int32_t ape_stream_load_i32(const int32_t* p) { return *p; }
static inline const void* ape_stream_load_ptr(const void* const* p) { return *p; }
static inline int ape_stream_find_chunk(const int32_t* cu, int n_chunks, int t) {
    int lo = 0, hi = n_chunks - 1;
    while (lo < hi) { const int mid = (lo + hi + 1) >> 1; if (cu[mid] <= t) lo = mid; else hi = mid - 1; }
    return lo;
}
#include "../paper_2502_05431_amd/csrc/ape_decode_stream.h"

using namespace ape;

struct View {
    const int32_t* cu;
    const void* const* k_chunks;
    const void* const* v_chunks;
    int n_chunks;
};

static long n_fail = 0, n_tiles = 0, n_cases = 0;
#define CHECK(cond, ...) do { if (!(cond)) { if (n_fail < 20) { printf("FAIL %s:%d: ", __FILE__, __LINE__); printf(__VA_ARGS__); printf("\n"); } ++n_fail; } } while (0)

constexpr long kStride = 8 * 256, kHead = 3 * 256;          // 8 KV heads, this workgroup's head = 3
constexpr uintptr_t kBaseK = (uintptr_t)1 << 44, kBaseV = (uintptr_t)1 << 45, kChunkSpan = (uintptr_t)1 << 34;

struct Table {
    std::vector<int32_t> cu;
    std::vector<const void*> k, v;
    View view() const { return View{cu.data(), k.data(), v.data(), (int)k.size()}; }
};

static Table make_table(const std::vector<int>& lens) {
    Table t;
    t.cu.push_back(0);
    for (size_t c = 0; c < lens.size(); ++c) {
        t.cu.push_back(t.cu.back() + lens[c]);
        t.k.push_back((const void*)(kBaseK + c * kChunkSpan));
        t.v.push_back((const void*)(kBaseV + c * kChunkSpan));
    }
    return t;
}

// Walks one wavefront's share [lo, hi) and marks the pooled tokens it delivers.
static void walk_ctx(const Table& tb, long lo, long hi, std::vector<int>& seen) {
    const View vw = tb.view();
    const long table_end = tb.cu.back();
    DecodeStream sm;
    sm.init_ctx(vw, lo, hi, kStride, kHead);
    long expect = lo;
    const char *kb, *vb;
    int nv;
    int guard = 0;
    while (sm.next(kb, vb, nv)) {
        ++n_tiles;
        if (++guard > 1 << 20) { CHECK(false, "stream does not end"); break; }
        CHECK(nv >= 1 && nv <= kDecodeTile, "tile of %d rows", nv);
        const uintptr_t ka = (uintptr_t)kb - kHead - kBaseK, va = (uintptr_t)vb - kHead - kBaseV;
        CHECK(ka == va, "K and V addresses disagree");
        const long c = (long)(ka / kChunkSpan), off = (long)(ka % kChunkSpan);
        CHECK(c >= 0 && c < vw.n_chunks, "chunk %ld outside the table", c);
        if (c < 0 || c >= vw.n_chunks) break;
        CHECK(off % kStride == 0, "row offset %ld is not a multiple of the stride", off);
        const long row = off / kStride, len = tb.cu[c + 1] - tb.cu[c];
        CHECK(row >= 0 && row + nv <= len, "rows [%ld, %ld) outside chunk %ld of %ld rows", row, row + nv, c, len);
        const long pooled = tb.cu[c] + row;
        CHECK(pooled == expect, "tile starts at token %ld, expected %ld", pooled, expect);
        for (int i = 0; i < nv; ++i)
            if (pooled + i < (long)seen.size()) ++seen[pooled + i];
        expect = pooled + nv;
    }
    const long want_end = lo < hi ? (hi < table_end ? hi : (lo < table_end ? table_end : lo)) : lo;
    CHECK(expect == want_end, "share [%ld, %ld) of a table of %ld tokens ended at %ld, expected %ld", lo, hi, table_end, expect, want_end);
}

static void run_ctx_case(const std::vector<int>& lens, long total_ctx, long split_len) {
    ++n_cases;
    const Table tb = make_table(lens);
    const long table_end = tb.cu.back();
    const long covered = total_ctx < table_end ? total_ctx : table_end;
    std::vector<int> seen(covered > 0 ? covered : 0, 0);
    const long n_splits = (total_ctx + split_len - 1) / split_len;
    for (long s = 0; s < n_splits + 1; ++s) {                 // one split past the end: empty
        const long t0 = s * split_len, t1 = total_ctx < t0 + split_len ? total_ctx : t0 + split_len;
        for (int w = 0; w < kDecodeWaves; ++w) {
            long lo, hi;
            decode_wave_share(t0, t1, w, lo, hi);
            if (t0 >= t1) CHECK(lo >= hi, "share of an empty split is not empty");
            walk_ctx(tb, lo, hi, seen);
        }
    }
    for (long i = 0; i < covered; ++i) CHECK(seen[i] == 1, "token %ld delivered %d times (split_len %ld, total %ld)", i, seen[i], split_len, total_ctx);
}

// explicit ranges, as the tree entry point passes them: consecutive, of any length, some empty
static void run_range_case(const std::vector<int>& lens, std::mt19937& rng) {
    ++n_cases;
    const Table tb = make_table(lens);
    const long total = tb.cu.back();
    std::vector<int> seen(total, 0);
    long t = 0;
    while (t < total) {
        long n = (long)(rng() % 5 == 0 ? 0 : 1 + rng() % 700);
        if (t + n > total) n = total - t;
        for (int w = 0; w < kDecodeWaves; ++w) {
            long lo, hi;
            decode_wave_share(t, t + n, w, lo, hi);
            walk_ctx(tb, lo, hi, seen);
        }
        t += n;
    }
    for (long i = 0; i < total; ++i) CHECK(seen[i] == 1, "token %ld delivered %d times (explicit ranges)", i, seen[i]);
}

static void run_plain_case(int np, int ns) {
    ++n_cases;
    std::vector<int> seen_p(np, 0), seen_s(ns, 0);
    const uintptr_t bk0 = kBaseK, bv0 = kBaseV, bk1 = kBaseK + kChunkSpan, bv1 = kBaseV + kChunkSpan;
    for (int w = 0; w < kDecodeWaves; ++w) {
        int pb, pe, sb, se;
        decode_plain_shares(np, ns, w, pb, pe, sb, se);
        CHECK(0 <= pb && pb <= pe && pe <= np && 0 <= sb && sb <= se && se <= ns, "shares out of range");
        DecodeStream sm;
        sm.init_plain((const char*)(bk0 + (long)pb * kStride + kHead), (const char*)(bv0 + (long)pb * kStride + kHead), pe - pb,
                      (const char*)(bk1 + (long)sb * kStride + kHead), (const char*)(bv1 + (long)sb * kStride + kHead), se - sb, kStride);
        const char *kb, *vb;
        int nv, guard = 0;
        while (sm.next(kb, vb, nv)) {
            ++n_tiles;
            if (++guard > 1 << 20) { CHECK(false, "stream does not end"); break; }
            CHECK(nv >= 1 && nv <= kDecodeTile, "tile of %d rows", nv);
            const uintptr_t ka = (uintptr_t)kb - kHead - kBaseK, va = (uintptr_t)vb - kHead - kBaseV;
            CHECK(ka == va, "K and V addresses disagree");
            const int seg = (int)(ka / kChunkSpan);
            const long row = (long)(ka % kChunkSpan) / kStride;
            CHECK(seg == 0 || seg == 1, "segment %d", seg);
            std::vector<int>& seen = seg == 0 ? seen_p : seen_s;
            CHECK(row >= 0 && row + nv <= (long)seen.size(), "rows [%ld, %ld) outside segment %d of %zu rows", row, row + nv, seg, seen.size());
            for (int i = 0; i < nv && row + i < (long)seen.size(); ++i) ++seen[row + i];
        }
    }
    for (int i = 0; i < np; ++i) CHECK(seen_p[i] == 1, "prefix row %d delivered %d times (np %d, ns %d)", i, seen_p[i], np, ns);
    for (int i = 0; i < ns; ++i) CHECK(seen_s[i] == 1, "own row %d delivered %d times (np %d, ns %d)", i, seen_s[i], np, ns);
}

int main() {
    std::mt19937 rng(20250205);
    const int pool[] = {0, 1, 2, 31, 32, 33, 63, 64, 65, 100, 127, 128, 129, 257, 512, 700, 1024, 2048, 3000};
    const long split_lens[] = {64, 128, 256, 512, 576, 1024, 2048, 4096};
    for (int it = 0; it < 400; ++it) {
        const int n = 1 + rng() % 12;
        std::vector<int> lens(n);
        for (int& l : lens) l = pool[rng() % (sizeof(pool) / sizeof(pool[0]))];
        long total = 0;
        for (int l : lens) total += l;
        for (long sl : split_lens) {
            run_ctx_case(lens, total, sl);
            if (it % 4 == 0) run_ctx_case(lens, total + 1 + rng() % 100, sl);       // the table holds fewer tokens than stated
            if (it % 4 == 1 && total > 1) run_ctx_case(lens, total - 1 - rng() % (total - 1), sl);   // ... or more
        }
        run_range_case(lens, rng);
    }
    run_ctx_case({5}, 0, 64);                                                       // no context at all
    run_ctx_case({0, 0, 0}, 0, 64);
    for (int np = 0; np <= 200; np += (np < 70 ? 1 : 13))
        for (int ns = 1; ns <= 300; ns += (ns < 70 ? 1 : 17)) run_plain_case(np, ns);
    printf("%ld cases; %ld tiles; %ld failed\n", n_cases, n_tiles, n_fail);
    return n_fail ? 1 : 0;
}
