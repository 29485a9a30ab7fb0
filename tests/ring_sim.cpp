// Host simulation of the scalar ring bookkeeping of the flash kernels (csrc/ape_ring.h): the
// control flow of run_blocks() in csrc/ape_flash_mfma.hip -- prologue, fast stretches, generic
// bodies -- with the MFMA work replaced by checks.  For every stream it verifies that
//   * every block is loaded exactly once, in stream order, from in-bounds addresses, into a slot
//     that no body still uses;
//   * body j finds block j-1, j and j+1 in the slots it reads, and the descriptors it is given
//     (valid rows, causal index) are those of blocks j and j+1;
//   * a fast body only ever meets full blocks that need no mask and issues only full blocks;
//   * every block is processed, and all wavefronts (which differ in their causal limits) execute
//     the same number of barriers.
// Build: g++ -O1 -std=c++17 [-fsanitize=address,undefined] ring_sim.cpp; exit status 0 = all streams pass.
#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <map>
#include <string>
#include <utility>
#include <vector>

#define APE_RING_FN inline
static inline int32_t ape_ring_load_i32(const int32_t* p) { return *p; }
static inline const void* ape_ring_load_ptr(const void* const* p) { return *p; }
static inline void ape_ring_load_chunk(const int32_t* cu_next, const void* const* kp, const void* const* vp, int32_t& c1, const void*& k, const void*& v) {
    c1 = *cu_next; k = *kp; v = *vp;
}
static inline int ape_ring_find_chunk(const int32_t* cu, int n_chunks, int t) {
    int lo = 0, hi = n_chunks - 1;
    while (lo < hi) { const int mid = (lo + hi + 1) >> 1; if (cu[mid] <= t) lo = mid; else hi = mid - 1; }
    return lo;
}
#include "../paper_2502_05431_amd/csrc/ape_ring.h"

using namespace ape;

struct Sim {
    std::map<const char*, int> block_of_ptr;                    // row-0 pointer of a block -> its index in the stream
    std::vector<int> ref_desc;                                  // descriptor of every block, from a plain walk
    std::vector<std::pair<const char*, const char*>> valid;     // valid K row ranges
    std::vector<int> slot_block;                                // which block each ring slot holds
    int next_to_issue = 0, barriers = 0, bodies = 0, fast = 0, static_bodies = 0;
    bool static_ring = false;                                   // run fast stretches as the wide prefill tile does
    std::string err;
    void fail(const std::string& m) { if (err.empty()) err = m; }
    void issue(const char* bk, int n_valid, long stride_b, int slot_off, int busy0, int busy1, int busy2) {
        for (int r = 0; r < n_valid; ++r) {
            const char* a = bk + (long)r * stride_b;
            bool ok = false;
            for (auto& v : valid) ok = ok || (a >= v.first && a + ROWB <= v.second);
            if (!ok) fail("load out of bounds");
        }
        auto it = block_of_ptr.find(bk);
        if (it == block_of_ptr.end()) { fail("load of an unknown block"); return; }
        if (it->second != next_to_issue) fail("blocks loaded out of order");
        if (n_valid != desc_n(ref_desc[it->second])) fail("loaded row count differs from the block's");
        const int slot = slot_off / SLOTB;
        if (slot == busy0 || slot == busy1 || slot == busy2) fail("load into a slot still in use, block " + std::to_string(it->second));
        slot_block[slot] = it->second;
        ++next_to_issue;
    }
};

template <int RING>
void run(Sim& sim, const Stream& ld0, int vis_lo) {
    constexpr int NF = RING - 3;
    const std::vector<int>& ref = sim.ref_desc;
    sim.slot_block.assign(RING, -1);
    if (ld0.rem == 0) { if (!ref.empty()) sim.fail("non-empty stream starts empty"); return; }
    RingPlan<RING> plan;
    plan.ld = ld0;
    plan.vis_lo = vis_lo;
    auto issue_next = [&](int slot_off) {
        const char *bk, *bv;
        const int d = plan.ld.take(bk, bv);
        sim.issue(bk, desc_n(d), plan.ld.stride_b, slot_off, -1, -1, -1);
        return d;
    };
    const int d0 = issue_next(0);
    int first[NF + 1];
    for (int i = 0; i <= NF; ++i) first[i] = 0;
    for (int i = 0; i < NF; ++i) first[i] = plan.ld.rem > 0 ? issue_next((i + 1) * SLOTB) : 0;
    sim.barriers++;
    plan.d_cur = d0;
    plan.d_nxt = first[0];
    for (int i = 0; i < NF; ++i) plan.fifo[i] = first[i + 1];
    plan.deep = NF >= 2 && plan.fifo[NF >= 2 ? NF - 2 : 0] != 0;
    plan.o_pv = (RING - 1) * SLOTB; plan.o_cur = 0; plan.o_nxt = SLOTB; plan.o_new = (RING - 2) * SLOTB;
    plan.piece(2);
    plan.piece(3);
    int pv_off = 0, j = 0;
    const int n_blocks = (int)ref.size();
    auto masked = [&](int d) { return plan.masked(d); };
    auto check_slots = [&](bool has_next) {
        if (sim.slot_block[plan.o_cur / SLOTB] != j) sim.fail("block j not in its slot at body " + std::to_string(j));
        if (has_next && sim.slot_block[plan.o_nxt / SLOTB] != j + 1) sim.fail("block j+1 not in its slot at body " + std::to_string(j));
        if (j > 0 && sim.slot_block[pv_off / SLOTB] != j - 1) sim.fail("block j-1 not in its slot at body " + std::to_string(j));
    };
    for (int guard = 0; guard < 1000000 && sim.err.empty(); ++guard) {
        const int n_fast = plan.fast_bodies();
        // the kernels' split of a stretch (wide prefill tile): bodies with run-time slots until the ring is
        // back at slot 0, then groups of RING bodies whose slots are compile-time constants and which
        // leave the plan's ring offsets and pv_off alone
        const FastSplit fs = sim.static_ring ? split_fast<RING>(n_fast, plan.o_cur / SLOTB, pv_off == plan.o_cur) : FastSplit{0, 0};
        for (int i = 0; i < n_fast && sim.err.empty(); ++i) {             // fast bodies
            if (j + 1 >= n_blocks) { sim.fail("fast body without a next block"); break; }
            sim.barriers++;
            const bool is_static = fs.supers > 0 && i >= fs.pre && i < fs.pre + fs.supers * RING;
            if (!is_static) {
                const int next_pv_off = plan.o_cur;
                check_slots(true);
                if (desc_n(ref[j]) != BLK || masked(ref[j])) sim.fail("fast body on a block that needs a mask, body " + std::to_string(j));
                sim.issue(plan.new_k, BLK, plan.ld.stride_b, plan.o_new, plan.o_cur / SLOTB, plan.o_nxt / SLOTB, j > 0 ? pv_off / SLOTB : -1);
                plan.fast_piece(0); plan.fast_piece(1); plan.fast_piece(2);
                pv_off = next_pv_off;
            } else {
                const int ph = (i - fs.pre) % RING;                        // the body's compile-time phase
                const int s_cur = ph, s_nxt = (ph + 1) % RING, s_pv = (ph + RING - 1) % RING, s_new = (ph + RING - 2) % RING;
                if (ph == 0 && (plan.o_cur != 0 || pv_off != (RING - 1) * SLOTB)) sim.fail("a group of static bodies does not start at slot 0, body " + std::to_string(j));
                if (sim.slot_block[s_cur] != j) sim.fail("static body: block j not in its slot, body " + std::to_string(j));
                if (sim.slot_block[s_nxt] != j + 1) sim.fail("static body: block j+1 not in its slot, body " + std::to_string(j));
                if (sim.slot_block[s_pv] != j - 1) sim.fail("static body: block j-1 not in its slot, body " + std::to_string(j));
                if (desc_n(ref[j]) != BLK || masked(ref[j])) sim.fail("fast body on a block that needs a mask, body " + std::to_string(j));
                sim.issue(plan.new_k, BLK, plan.ld.stride_b, s_new * SLOTB, s_cur, s_nxt, s_pv);
                plan.fast_piece(0); plan.fast_piece(1);                    // (piece 2, the ring's turn, is left out)
                sim.static_bodies++;
            }
            ++j; sim.bodies++; sim.fast++;
        }
        if (n_fast > 0) plan.finish_fast(n_fast);
        if (!sim.err.empty()) break;
        // generic body
        const int d_nxt = plan.d_nxt;
        if (d_nxt != 0) sim.barriers++;
        const int next_pv_off = plan.o_cur;
        check_slots(d_nxt != 0);
        if (j >= n_blocks) { sim.fail("more bodies than blocks"); break; }
        if (plan.d_cur != ref[j]) sim.fail("descriptor of block j wrong at body " + std::to_string(j));
        if (plan.d_nxt != (j + 1 < n_blocks ? ref[j + 1] : 0)) sim.fail("descriptor of block j+1 wrong at body " + std::to_string(j));
        if (plan.cur_masked != masked(ref[j])) sim.fail("mask flag wrong at body " + std::to_string(j));
        if (plan.d_new != 0)
            sim.issue(plan.new_k, desc_n(plan.d_new), plan.ld.stride_b, plan.o_new, plan.o_cur / SLOTB, d_nxt != 0 ? plan.o_nxt / SLOTB : -1,
                      j > 0 ? pv_off / SLOTB : -1);
        if (d_nxt != 0) { plan.piece(0); plan.piece(1); plan.piece(2); plan.piece(3); }
        pv_off = next_pv_off; ++j; sim.bodies++;
        if (d_nxt == 0) break;
    }
    if (sim.err.empty() && j != n_blocks) sim.fail("processed " + std::to_string(j) + " of " + std::to_string(n_blocks) + " blocks");
    if (sim.err.empty() && sim.next_to_issue != n_blocks) sim.fail("loaded " + std::to_string(sim.next_to_issue) + " of " + std::to_string(n_blocks) + " blocks");
}

static void walk(Stream ld, Sim& sim) {
    int idx = 0;
    while (ld.rem > 0) {
        const char *bk, *bv;
        const int d = ld.take(bk, bv);
        sim.block_of_ptr[bk] = idx++;
        sim.ref_desc.push_back(d);
    }
}

struct Tally { int cases = 0, failed = 0, fast = 0, bodies = 0, static_bodies = 0; };

template <typename MakeStream>
static void run_case(Tally& t, const char* what, MakeStream make, const std::vector<std::pair<const char*, const char*>>& valid,
                     const std::vector<int>& vis_los, int expect_rows) {
    // (ring 6 twice: the second time with fast stretches split as the wide prefill tile splits them)
    for (int variant = 0; variant < 4; ++variant) {
        const int ring = variant == 0 ? 5 : variant == 3 ? 8 : 6;
        int barriers = -1;
        for (int vis_lo : vis_los) {
            Sim sim; sim.valid = valid; sim.static_ring = variant == 2;
            Stream ld = make();
            walk(ld, sim);
            int rows = 0; for (int d : sim.ref_desc) rows += desc_n(d);
            if (rows != expect_rows) sim.fail("stream delivers " + std::to_string(rows) + " rows, expected " + std::to_string(expect_rows));
            if (ring == 5) run<5>(sim, ld, vis_lo); else if (ring == 6) run<6>(sim, ld, vis_lo); else run<8>(sim, ld, vis_lo);
            if (sim.err.empty() && barriers >= 0 && sim.barriers != barriers) sim.fail("wavefronts with different causal limits execute different numbers of barriers");
            barriers = sim.barriers;
            ++t.cases; t.fast += sim.fast; t.bodies += sim.bodies; t.static_bodies += sim.static_bodies;
            if (!sim.err.empty() && t.failed++ < 20) std::printf("%s ring=%d vis_lo=%d: %s\n", what, ring, vis_lo, sim.err.c_str());
        }
    }
}

int main() {
    Tally t;
    const long stride_b = 2048;
    std::vector<char> buf((size_t)1 << 26);
    const char* base = buf.data() + 4096;
    char what[256];
    // sequence streams (encode tiles, the prefix+self split): a plain segment, then a causal one
    for (int np : {0, 5, 7, 31, 32, 33, 40, 64, 100})
        for (int nc = 1; nc <= 4200; nc += (nc < 70 ? 1 : nc < 700 ? 29 : 1171)) {
            const char* kp = base; const char* kc = base + (long)(np + 8) * stride_b + (1 << 19);
            std::vector<std::pair<const char*, const char*>> valid = {{kp, kp + (long)np * stride_b}, {kc, kc + (long)nc * stride_b}};
            std::snprintf(what, sizeof what, "seq prefix=%d causal=%d", np, nc);
            run_case(t, what, [&] { Stream ld; ld.init_seq(kp, kp + (1 << 25), np, kc, kc + (1 << 25), nc, stride_b); return ld; }, valid,
                     {0, 8, 24, 31, 32, 48, 63, 64, 100, 200, 399, 699, 2500, 5000}, np + nc);
        }
    // context streams: ranges of the pooled contexts through a chunk table
    const std::vector<std::vector<int>> tables = {{64, 64}, {100, 1, 65, 300, 31}, {2048, 2048, 2048, 2048}, {257, 255}, {512, 512, 512}, {130},
                                                  {32, 0, 0, 64, 1, 0, 33}, {256, 256, 256, 256, 256, 256, 256, 256}, {1, 1, 1, 1, 1}};
    // gap 0: the contexts lie back to back (a packed cache), where a run of full blocks continues
    // across context boundaries; otherwise they are apart
    for (long gap : {8192L, 0L})
    for (size_t v = 0; v < tables.size(); ++v) {
        const std::vector<int>& lens = tables[v];
        std::vector<int32_t> cu(1, 0);
        for (int l : lens) cu.push_back(cu.back() + l);
        std::vector<const void*> kc, vc;
        std::vector<std::pair<const char*, const char*>> valid;
        long off = 0;
        for (int l : lens) { kc.push_back(base + off); vc.push_back(base + (1 << 25) + off); valid.push_back({base + off, base + off + (long)l * stride_b}); off += (long)l * stride_b + gap; }
        const int total = cu.back();
        for (int split_len : {64, 128, 320, 1024, 8192})
            for (int t0 = 0; t0 < total; t0 += split_len) {
                const int t1 = std::min(total, t0 + split_len);
                std::snprintf(what, sizeof what, "ctx table=%zu split_len=%d t0=%d", v, split_len, t0);
                run_case(t, what, [&] { Stream ld; ld.init_ctx(cu.data(), kc.data(), vc.data(), (int)lens.size(), t0, t1, stride_b, 0); return ld; }, valid,
                         {0}, t1 - t0);
            }
        // per-context splits (tree merge): every context cut into `sub` runs of its own, the last
        // one open-ended; empty runs never reach the block loop
        const int max_len = *std::max_element(lens.begin(), lens.end());
        for (int sub : {1, 2, 3, 5})
            for (size_t c = 0; c < lens.size(); ++c)
                for (int j = 0; j < sub; ++j) {
                    const int len = ((max_len + sub - 1) / sub + 63) / 64 * 64;
                    const int c0 = cu[c], c1 = cu[c + 1];
                    const int t0 = std::min(c1, c0 + j * len);
                    const int t1 = j == sub - 1 ? c1 : std::min(c1, t0 + len);
                    if (t0 >= t1) continue;
                    std::snprintf(what, sizeof what, "ctx table=%zu context=%zu sub=%d/%d", v, c, j, sub);
                    run_case(t, what, [&] { Stream ld; ld.init_ctx(cu.data(), kc.data(), vc.data(), (int)lens.size(), t0, t1, stride_b, 0); return ld; }, valid,
                             {0}, t1 - t0);
                }
    }
    std::printf("%d streams, %d failed; %d of %d bodies fast; %d in groups with compile-time slots\n", t.cases, t.failed, t.fast, t.bodies, t.static_bodies);
    return t.failed != 0;
}
