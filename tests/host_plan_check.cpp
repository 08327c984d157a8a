// Host check of the launch plans klay_build hands to the kernels, with no GPU: random DAGs are
// layerized with many option sets and every pass plan (main rows as tasks, segments of split rows,
// combine lists) is executed here in plain C++ on integer "values", in the same order of steps the
// device kernels take, and compared with the sums over the plain per-layer index vectors
// (paper Section 4: E_l = N_{l-1}[S_l], N_l = scatter(E_l, R_l)).  Built with the address and
// undefined-behaviour sanitizers by tests/test_host_plans.py.
#include <cstdio>
#include <cstdlib>
#include <random>
#include <string>
#include <vector>

#include "../paper_2410_11415_amd/csrc/layerize.h"

using klay::PassPlan;
using u64 = unsigned long long;

static u64 mix(u64 x) { x += 0x9E3779B97F4A7C15ull; x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull; x = (x ^ (x >> 27)) * 0x94D049BB133111EBull; return x ^ (x >> 31); }
static constexpr uint32_t kMask = klay::kRowFlag - 1u;

#define CHECK(cond, ...) do { if (!(cond)) { std::printf("FAILED %s:%d: ", __FILE__, __LINE__); std::printf(__VA_ARGS__); std::printf("\n"); std::exit(1); } } while (0)

// value of source row i, and weight tag of an entry (so that a wrong weighted flag changes the sum)
static u64 val(int64_t i) { return mix((u64)i); }
static u64 entry(uint32_t id) { return val(id & kMask) * ((id & klay::kWeightedEdge) ? 3u : 1u); }

// the walk of the streaming kernel over a task list: rows advance on the end-of-row bit
static void walk_tasks(const PassPlan& p, const std::vector<int32_t>& tasks, int n_tasks, int64_t n_src,
                       std::vector<u64>& out, std::vector<int>& written, int64_t row_shift) {
    CHECK((int)tasks.size() == 2 * (n_tasks + 1), "task array size");
    for (int t = 0; t < n_tasks; ++t) {
        int row = tasks[2 * t], j = tasks[2 * t + 1];
        const int row_end = tasks[2 * t + 2], e1 = tasks[2 * t + 3];
        CHECK(j < e1 && row < row_end, "empty task %d", t);
        u64 acc = 0;
        for (; j < e1; ++j) {
            const uint32_t id = p.idx[(size_t)j];
            if (id == klay::kSkipRow) { CHECK(acc == 0, "skip entry inside a row"); ++row; continue; }
            CHECK((int64_t)(id & kMask) < n_src, "source %u out of range %lld", id & kMask, (long long)n_src);
            acc += entry(id);
            if (id & klay::kLastEdge) {
                CHECK(row - row_shift >= 0 && row - row_shift < (int64_t)out.size(), "row out of range");
                out[(size_t)(row - row_shift)] = acc; ++written[(size_t)(row - row_shift)];
                acc = 0; ++row;
            }
        }
        CHECK(acc == 0, "task %d ends inside a row", t);
        CHECK(row == row_end, "task %d covers rows up to %d, next task starts at %d", t, row, row_end);
    }
}

// the walk of the generic kernel: rows by ptr
static void walk_rows(const PassPlan& p, int row_begin, int row_end, int64_t n_src, std::vector<u64>& main_out,
                      std::vector<int>& main_written, std::vector<u64>& seg_out, std::vector<int>& seg_written) {
    for (int row = row_begin; row < row_end; ++row) {
        const int beg = p.ptr[(size_t)row], end = p.ptr[(size_t)row + 1];
        CHECK(end > beg, "empty row %d", row);
        if (p.idx[(size_t)beg] == klay::kSkipRow) { CHECK(end == beg + 1 && row < p.n_main, "skip row shape"); continue; }
        u64 acc = 0;
        for (int j = beg; j < end; ++j) {
            const uint32_t id = p.idx[(size_t)j];
            CHECK((int64_t)(id & kMask) < n_src, "source out of range");
            CHECK(((id & klay::kLastEdge) != 0) == (j == end - 1), "end-of-row bit of row %d", row);
            acc += entry(id);
        }
        if (row < p.n_main) { main_out[(size_t)row] = acc; ++main_written[(size_t)row]; }
        else { seg_out[(size_t)(row - p.n_main)] = acc; ++seg_written[(size_t)(row - p.n_main)]; }
    }
}

// runs one plan both ways and compares with `want` (one value per output row)
// `left_out` (optional, a byte per row): rows the plan must not write (the fused rows of LayerPlan::fwd_kept)
static void check_plan(const PassPlan& p, int64_t n_out, int64_t n_src, const std::vector<u64>& want, const char* what,
                       const std::vector<uint32_t>* row_bits = nullptr, const std::vector<uint8_t>* left_out = nullptr) {
    CHECK(p.n_main == n_out, "%s: n_main", what);
    // the row flag sits on the last entry of exactly the flagged rows (a split row: on the last entry of its
    // combine list) and nowhere else
    {
        auto flagged = [&](int64_t r) { return row_bits && (((*row_bits)[(size_t)r >> 5] >> (r & 31)) & 1u); };
        for (int64_t r = 0; r < (int64_t)p.n_main + p.n_seg; ++r)
            for (int j = p.ptr[(size_t)r]; j < p.ptr[(size_t)r + 1]; ++j) {
                const uint32_t id = p.idx[(size_t)j];
                if (id == klay::kSkipRow) continue;
                const bool expect = r < p.n_main && j == p.ptr[(size_t)r + 1] - 1 && flagged(r);
                CHECK(((id & klay::kRowFlag) != 0) == expect, "%s: row flag of row %lld", what, (long long)r);
            }
        for (int h = 0; h < p.n_heavy; ++h)
            for (int j = p.comb_ptr[(size_t)h]; j < p.comb_ptr[(size_t)h + 1]; ++j) {
                const bool expect = j == p.comb_ptr[(size_t)h + 1] - 1 && flagged(p.comb_row[(size_t)h]);
                CHECK(((p.comb_idx[(size_t)j] & klay::kRowFlag) != 0) == expect, "%s: row flag of split row %d", what, h);
            }
    }
    CHECK((int64_t)p.ptr.size() == (int64_t)p.n_main + p.n_seg + 1, "%s: ptr size", what);
    const int64_t entries = p.ptr.back();
    CHECK((int64_t)p.idx.size() == entries + klay::kIdxPad, "%s: idx size", what);
    for (int i = 0; i < klay::kIdxPad; ++i) CHECK(p.idx[(size_t)entries + i] == 0u, "%s: idx padding", what);
    CHECK((int64_t)p.seg_owner.size() == p.n_seg && (int64_t)p.comb_row.size() == p.n_heavy, "%s: sizes", what);
    if (p.n_heavy > 0) CHECK((int64_t)p.comb_idx.size() == (int64_t)p.n_seg + klay::kIdxPad, "%s: comb_idx size", what);
    else CHECK(p.n_seg == 0, "%s: segments without split rows", what);
    for (int variant = 0; variant < 2; ++variant) {
        std::vector<u64> out((size_t)n_out, 0), seg((size_t)p.n_seg, 0);
        std::vector<int> wr((size_t)n_out, 0), swr((size_t)p.n_seg, 0);
        if (variant == 0) {
            walk_tasks(p, p.tasks, p.n_tasks, n_src, out, wr, 0);
            if (p.n_seg > 0) walk_tasks(p, p.seg_tasks, p.n_seg_tasks, n_src, seg, swr, p.n_main);
        } else {
            walk_rows(p, 0, p.n_main + p.n_seg, n_src, out, wr, seg, swr);
        }
        for (int s = 0; s < p.n_seg; ++s) CHECK(swr[(size_t)s] == 1, "%s: segment %d written %d times", what, s, swr[(size_t)s]);
        std::vector<int> seg_used((size_t)p.n_seg, 0);
        for (int h = 0; h < p.n_heavy; ++h) {
            const int row = p.comb_row[(size_t)h];
            CHECK(row >= 0 && row < n_out && wr[(size_t)row] == 0, "%s: split row %d also written by the main pass", what, row);
            u64 acc = 0;
            for (int j = p.comb_ptr[(size_t)h]; j < p.comb_ptr[(size_t)h + 1]; ++j) {
                const uint32_t s = p.comb_idx[(size_t)j] & kMask;
                CHECK((int)s < p.n_seg && p.seg_owner[(size_t)s] == row, "%s: segment %u of split row %d", what, s, row);
                acc += seg[(size_t)s]; ++seg_used[(size_t)s];
            }
            out[(size_t)row] = acc; ++wr[(size_t)row];
        }
        for (int s = 0; s < p.n_seg; ++s) CHECK(seg_used[(size_t)s] == 1, "%s: segment %d combined %d times", what, s, seg_used[(size_t)s]);
        for (int64_t i = 0; i < n_out; ++i) {
            if (left_out && (*left_out)[(size_t)i]) { CHECK(wr[(size_t)i] == 0, "%s: row %lld is written", what, (long long)i); continue; }
            CHECK(wr[(size_t)i] == 1, "%s: row %lld written %d times (variant %d)", what, (long long)i, wr[(size_t)i], variant);
            CHECK(out[(size_t)i] == want[(size_t)i], "%s: row %lld value (variant %d)", what, (long long)i, variant);
        }
    }
}

// the walk of the persistent kernels over a chunked plan: each of the 16 waves streams through its run
// of lines, one word per lane; the end-of-chunk bit (the same in all 64 words of a line) closes the 64
// rows of the chunk in hand, and the wave's next chunk is 16 chunks further; padding words add nothing
static void check_slab(const klay::SlabPlan& sp, int64_t n_out, int64_t n_src, const std::vector<u64>& want, const char* what,
                       const std::vector<uint32_t>* row_bits = nullptr) {
    const int64_t chunks = (n_out + 63) / 64;
    CHECK(sp.wave_line[0] == 0 && (int64_t)sp.ent.size() == (int64_t)sp.wave_line[klay::kSlabWaves] * 64, "%s: sizes", what);
    std::vector<int> written((size_t)n_out, 0);
    for (int w = 0; w < klay::kSlabWaves; ++w) {
        int64_t q = w;
        std::vector<u64> acc(64, 0);
        std::vector<int> ended(64, 0);
        CHECK(sp.wave_line[w + 1] >= sp.wave_line[w], "%s: run bounds", what);
        CHECK((sp.wave_line[w + 1] - sp.wave_line[w]) % klay::kSlabBlock == 0, "%s: run is not a whole number of blocks", what);
        for (int64_t line = sp.wave_line[w]; line < sp.wave_line[w + 1]; ++line) {
            const uint32_t* e = sp.ent.data() + (size_t)line * 64;
            if (q >= chunks) {       // lines that fill the run up to a whole block: padding only, no end-of-chunk bit
                for (int lane = 0; lane < 64; ++lane) CHECK((int64_t)e[lane] == n_src, "%s: filler line of wave %d", what, w);
                continue;
            }
            for (int lane = 0; lane < 64; ++lane) {
                CHECK((e[lane] & klay::kLastEdge) == (e[0] & klay::kLastEdge), "%s: end-of-chunk bit differs within a line", what);
                {   // the row flag sits on the word a lane holds when its chunk closes, for flagged rows only
                    const int64_t r = q * 64 + lane;
                    const bool expect = (e[0] & klay::kLastEdge) && row_bits && r < n_out && (((*row_bits)[(size_t)r >> 5] >> (r & 31)) & 1u);
                    CHECK(((e[lane] & klay::kRowFlag) != 0) == expect, "%s: row flag of row %lld", what, (long long)r);
                }
                const uint32_t src = e[lane] & kMask;
                if ((int64_t)src == n_src) { CHECK(!(e[lane] & klay::kWeightedEdge), "%s: flag on padding", what); ended[(size_t)lane] = 1; continue; }
                CHECK(!ended[(size_t)lane], "%s: source after padding", what);
                CHECK(q * 64 + lane < n_out, "%s: source in a lane past the last row", what);
                CHECK((int64_t)src < n_src, "%s: source out of range", what);
                acc[(size_t)lane] += entry(e[lane] & ~klay::kLastEdge);
            }
            if (e[0] & klay::kLastEdge) {
                for (int lane = 0; lane < 64; ++lane) {
                    const int64_t r = q * 64 + lane;
                    if (r < n_out) { CHECK(acc[(size_t)lane] == want[(size_t)r], "%s: row %lld value", what, (long long)r); ++written[(size_t)r]; }
                    acc[(size_t)lane] = 0; ended[(size_t)lane] = 0;
                }
                q += klay::kSlabWaves;
            }
        }
        CHECK(q >= chunks && q < chunks + klay::kSlabWaves, "%s: wave %d ends at chunk %lld of %lld", what, w, (long long)q, (long long)chunks);
    }
    for (int64_t r = 0; r < n_out; ++r) CHECK(written[(size_t)r] == 1, "%s: row %lld closed %d times", what, (long long)r, written[(size_t)r]);
}

int main(int argc, char** argv) {
    const int trials = argc > 1 ? std::atoi(argv[1]) : 120;
    std::mt19937_64 rng(12345);
    long plans = 0, fused_plans = 0, b0_seen[3] = {0, 0, 0};
    for (int trial = 0; trial < trials; ++trial) {
        const int V = 1 + (int)(rng() % 12), nl = 2 * V;
        const int ng = 1 + (int)(rng() % 400);
        const int N = nl + 2 + ng;
        std::vector<uint8_t> type((size_t)N);
        std::vector<int32_t> lit((size_t)N, 0), idx;
        std::vector<int64_t> ptr((size_t)N + 1, 0);
        for (int v = 0; v < V; ++v) { type[2 * v] = 0; lit[2 * v] = v + 1; type[2 * v + 1] = 0; lit[2 * v + 1] = -(v + 1); }
        type[(size_t)nl] = 3; type[(size_t)nl + 1] = 4;
        for (int g = 0; g < ng; ++g) {
            const int id = nl + 2 + g;
            type[(size_t)id] = (uint8_t)(1 + rng() % 2);
            const int k = 1 + (int)(rng() % (trial % 5 == 0 ? 150 : 5));
            std::vector<int> kids;
            for (int j = 0; j < k; ++j) {
                // a few hub nodes give rows of high fan-out
                const int c = (rng() % 4 == 0) ? (int)(rng() % (nl < 6 ? nl : 6)) : (int)(rng() % id);
                bool dup = false;
                for (int x : kids) dup |= x == c;
                if (!dup) kids.push_back(c);
            }
            for (int c : kids) idx.push_back(c);
            ptr[(size_t)id + 1] = (int64_t)idx.size();
        }
        for (int i = 0; i < nl + 2; ++i) ptr[(size_t)i + 1] = 0;
        for (int g = 0; g < ng; ++g) if (ptr[(size_t)nl + 2 + g + 1] < ptr[(size_t)nl + 2 + g]) ptr[(size_t)nl + 2 + g + 1] = ptr[(size_t)nl + 2 + g];
        const int R = 1 + (int)(rng() % 4);
        std::vector<int32_t> roots((size_t)R);
        for (auto& r : roots) r = (int32_t)(rng() % N);
        for (int mode = 0; mode < 8; ++mode) {
            klay::Options o;
            o.alias_chains = mode & 1; o.no_merge = mode & 2; o.no_reorder = mode & 4;
            o.no_tail = (rng() % 4) == 0;
            o.tail_rows_cap = (rng() % 3) == 0 ? 0 : 2 + (int)(rng() % 12);
            o.heavy_fan = 1 + (int)(rng() % 40); o.min_segment = 1 + (int)(rng() % 8);
            klay::CircuitPlan plan;
            std::string err;
            const int st = klay::layerize(V, N, type.data(), lit.data(), ptr.data(), idx.data(), R, roots.data(), o, plan, err);
            if (st == 1) continue;                  // a repeated literal child after leaf merging: rejected input
            CHECK(st == 0, "layerize status %d: %s", st, err.c_str());
            const int L = plan.num_layers;
            const int B0 = plan.alias_top;
            CHECK(B0 >= 0 && B0 <= L && plan.alias == (B0 > 0), "alias_top %d of %d layers", B0, L);
            if (!o.alias_chains) CHECK(B0 == 0, "chains asked for");
            if (o.alias_chains && o.no_tail) CHECK(B0 == L, "no persistent top: padding-free throughout");
            ++b0_seen[B0 == 0 ? 0 : (B0 == L ? 2 : 1)];
            // layers above B0: edges to the layer directly below, reverse plans layer by layer
            for (int l = B0 + 1; l <= L; ++l) {
                const klay::LayerPlan& lay = plan.layers[(size_t)l];
                const int64_t nb = plan.layers[(size_t)l - 1].n;
                std::vector<u64> fwd((size_t)lay.n, 0), bwd((size_t)nb, 0);
                for (int64_t r = 0; r < lay.n; ++r) {
                    const bool weighted = (l % 2 == 0) && lay.row_ptr[(size_t)r + 1] - lay.row_ptr[(size_t)r] > 1;
                    for (int j = lay.row_ptr[(size_t)r]; j < lay.row_ptr[(size_t)r + 1]; ++j) {
                        CHECK(lay.child[(size_t)j] >= 0 && lay.child[(size_t)j] < nb, "child position in the layer below");
                        fwd[(size_t)r] += val(lay.child[(size_t)j]);
                        bwd[(size_t)lay.child[(size_t)j]] += val(r) * (weighted ? 3u : 1u);
                    }
                }
                check_plan(lay.fwd, lay.n, nb, fwd, "forward plan"); ++plans;
                check_plan(lay.bwd, nb, lay.n, bwd, "backward plan", (l % 2 == 1 && l >= 3) ? &plan.layers[(size_t)l - 1].multi : nullptr); ++plans;
                CHECK(!lay.tail_bwd_ok || lay.tail_fwd_ok, "reverse persistent plan without the forward one");
                if (lay.tail_fwd_ok) { check_slab(lay.slab_fwd, lay.n, nb, fwd, "persistent forward plan"); ++plans; }
                if (lay.tail_bwd_ok) { check_slab(lay.slab_bwd, nb, lay.n, bwd, "persistent reverse plan",
                                                  (l % 2 == 1 && l >= 3) ? &plan.layers[(size_t)l - 1].multi : nullptr); ++plans; }
            }
            for (int l = 1; l <= L; ++l) {
                const klay::LayerPlan& lay = plan.layers[(size_t)l];
                for (int64_t r = 0; r < lay.n; ++r)
                    CHECK(((lay.multi[(size_t)r >> 5] >> (r & 31)) & 1u) == (lay.row_ptr[(size_t)r + 1] - lay.row_ptr[(size_t)r] > 1 ? 1u : 0u), "multi-child bit");
                if (plan.tail_first > 0 && l >= plan.tail_first) CHECK(lay.tail_fwd_ok && l > B0, "candidate suffix");
                if (plan.tail_bwd_first > 0 && l >= plan.tail_bwd_first) CHECK(lay.tail_bwd_ok && plan.tail_bwd_first >= plan.tail_first, "reverse candidate suffix");
                if (l < B0) for (int64_t r = 0; r < lay.n; ++r) CHECK(!lay.is_pad[(size_t)r], "chain node below the boundary layer");
            }
            if (B0 > 0) {
                // layers up to B0: edges name rows of the whole buffer; reverse plans of the rows below B0 gather
                // from parents in any layer up to B0
                const int64_t NR = plan.row0[(size_t)B0];
                std::vector<u64> adj((size_t)NR, 0);
                for (int l = 1; l <= B0; ++l) {
                    const klay::LayerPlan& lay = plan.layers[(size_t)l];
                    std::vector<u64> fwd((size_t)lay.n, 0);
                    for (int64_t r = 0; r < lay.n; ++r) {
                        const bool weighted = (l % 2 == 0) && lay.row_ptr[(size_t)r + 1] - lay.row_ptr[(size_t)r] > 1;
                        for (int j = lay.row_ptr[(size_t)r]; j < lay.row_ptr[(size_t)r + 1]; ++j) {
                            const int32_t ch = lay.child[(size_t)j];
                            CHECK(ch >= 0 && ch < plan.row0[(size_t)l], "aliased child must sit in a lower layer");
                            fwd[(size_t)r] += val(ch);
                            adj[(size_t)ch] += val(plan.row0[(size_t)l] + r) * (weighted ? 3u : 1u);
                        }
                    }
                    check_plan(lay.fwd, lay.n, plan.row0[(size_t)l], fwd, "alias forward plan"); ++plans;
                }
                // Fused AND rows: fwd_kept is fwd without them; fwd2 of the OR layers reads, in place of a fused
                // row, that row's children as one group (the entry that closes a group counts three times here,
                // like a weighted one, so that a misplaced group end changes the sum).
                std::vector<uint8_t> is_fused((size_t)NR, 0);
                int64_t n_fused = 0;
                for (int l = 1; l < B0; l += 2) {
                    const klay::LayerPlan& lay = plan.layers[(size_t)l];
                    if (lay.n_fused == 0) { CHECK(lay.fwd_kept.ptr.empty(), "fwd_kept without fused rows"); continue; }
                    CHECK(lay.n_fused <= lay.n, "fused row count");
                    if (lay.n_fused == lay.n) { CHECK(lay.fwd_kept.ptr.empty(), "fwd_kept with nothing to evaluate"); }
                    std::vector<uint8_t> out((size_t)lay.n, 0);
                    std::vector<u64> fwd((size_t)lay.n, 0);
                    int64_t seen = 0;
                    std::vector<uint8_t> split_kept((size_t)lay.n, 0);
                    for (int32_t row : lay.fwd_kept.comb_row) split_kept[(size_t)row] = 1;
                    for (int64_t r = 0; r < lay.n; ++r) {
                        // a fused row: a skip entry in fwd_kept that no combine list of fwd_kept writes
                        const bool skipped = lay.n_fused == lay.n ||
                            (lay.fwd_kept.idx[(size_t)lay.fwd_kept.ptr[(size_t)r]] == klay::kSkipRow && !split_kept[(size_t)r]);
                        out[(size_t)r] = skipped;
                        seen += skipped;
                        is_fused[(size_t)(plan.row0[(size_t)l] + r)] = skipped;
                        for (int j = lay.row_ptr[(size_t)r]; j < lay.row_ptr[(size_t)r + 1]; ++j) fwd[(size_t)r] += val(lay.child[(size_t)j]);
                        if (skipped) {
                            int64_t gates = 0;
                            for (int j = lay.row_ptr[(size_t)r]; j < lay.row_ptr[(size_t)r + 1]; ++j) gates += lay.child[(size_t)j] >= plan.row0[1];
                            CHECK(gates <= 1, "a fused row has more than one child that is not a leaf");
                        }
                    }
                    CHECK(seen == lay.n_fused, "fused rows of layer %d: %lld counted, %lld marked", l, (long long)lay.n_fused, (long long)seen);
                    n_fused += seen;
                    if (lay.n_fused < lay.n) { check_plan(lay.fwd_kept, lay.n, plan.row0[(size_t)l], fwd, "forward plan without the fused rows", nullptr, &out); ++plans; }
                }
                CHECK(n_fused == plan.num_fused, "fused rows in total");
                for (int l = 2; l <= B0; l += 2) {
                    const klay::LayerPlan& lay = plan.layers[(size_t)l];
                    bool reads_fused = false;
                    std::vector<u64> want((size_t)lay.n, 0);
                    for (int64_t r = 0; r < lay.n; ++r)
                        for (int j = lay.row_ptr[(size_t)r]; j < lay.row_ptr[(size_t)r + 1]; ++j) {
                            const int32_t ch = lay.child[(size_t)j];
                            if (!is_fused[(size_t)ch]) { want[(size_t)r] += 3u * val(ch); continue; }
                            reads_fused = true;
                            // the fused child's own children; the last of them closes the group
                            int a = 1;
                            while (plan.row0[(size_t)a + 1] <= ch) ++a;
                            const klay::LayerPlan& al = plan.layers[(size_t)a];
                            const int64_t ar = ch - plan.row0[(size_t)a];
                            for (int jj = al.row_ptr[(size_t)ar]; jj < al.row_ptr[(size_t)ar + 1]; ++jj)      // (child lists are sorted)
                                want[(size_t)r] += val(al.child[(size_t)jj]) * (jj == al.row_ptr[(size_t)ar + 1] - 1 ? 3u : 1u);
                        }
                    CHECK(reads_fused == !lay.fwd2.ptr.empty(), "fwd2 of layer %d", l);
                    if (reads_fused) {
                        check_plan(lay.fwd2, lay.n, plan.row0[(size_t)l], want, "fused forward plan"); ++plans; fused_plans++;
                        // no group is cut by the end of a row or of a segment
                        for (size_t j = 0; j + klay::kIdxPad < lay.fwd2.idx.size(); ++j) {
                            const uint32_t id = lay.fwd2.idx[j];
                            if (id != klay::kSkipRow && (id & klay::kLastEdge)) CHECK((id & klay::kGroupEnd) != 0, "a group of entries runs past the end of its row (layer %d, entry %zu of %zu, %d main rows, %d segments, main entries %d)", l, j, lay.fwd2.idx.size(), lay.fwd2.n_main, lay.fwd2.n_seg, lay.fwd2.ptr[(size_t)lay.fwd2.n_main]);
                        }
                    }
                }
                for (int l = 0; l < B0; ++l) {
                    const int64_t a = plan.row0[(size_t)l], n = plan.layers[(size_t)l].n;
                    std::vector<u64> want(adj.begin() + a, adj.begin() + a + n);
                    check_plan(plan.layers[(size_t)l + 1].bwd, n, plan.row0[(size_t)B0 + 1], want, "alias backward plan",
                               (l % 2 == 0 && l >= 2) ? &plan.layers[(size_t)l].multi : nullptr); ++plans;
                }
            }
            // every root reads a row of the top layer
            for (int r = 0; r < R; ++r) CHECK(plan.root_pos[(size_t)r] >= 0 && plan.root_pos[(size_t)r] < plan.layers[(size_t)L].n, "root position");
        }
    }
    CHECK(b0_seen[0] > 0 && b0_seen[1] > 0 && b0_seen[2] > 0, "boundary layer cases seen: %ld %ld %ld", b0_seen[0], b0_seen[1], b0_seen[2]);
    CHECK(fused_plans > 0, "no fused forward plan was built");
    std::printf("ok: %ld plans checked (%ld fused forward plans)\n", plans, fused_plans);
    return 0;
}
