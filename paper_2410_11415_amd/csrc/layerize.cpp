// Host-side layerization and tensorization (paper Section 3.1 Eq. 2, Section 3.2, Alg. 2, Alg. 3).
#include "layerize.h"

#include <algorithm>
#include <climits>
#include <cmath>
#include <numeric>
#include <unordered_map>

namespace klay {

namespace {
// task size bounds (entries per wave task); overridable at compile time for tuning
#ifndef KLAY_TASK_MIN
#define KLAY_TASK_MIN 8
#endif
#ifndef KLAY_TASK_MAX
#define KLAY_TASK_MAX 32
#endif
#ifndef KLAY_TASK_DIV
#define KLAY_TASK_DIV 32768
#endif
constexpr int64_t kLatencyBoundEntries = 200000;     // see make_pass_plan
constexpr int64_t kTaskMin = KLAY_TASK_MIN, kTaskMax = KLAY_TASK_MAX, kTaskDiv = KLAY_TASK_DIV;
enum : uint8_t { T_LIT = 0, T_AND = 1, T_OR = 2, T_TRUE = 3, T_FALSE = 4 };
constexpr int ST_OK = 0, ST_INVAL = 1, ST_CYCLE = 2;

// Segment length for a split row of k sources: about sqrt(k), so that the segment pass and the combine
// pass both see rows of that length, but at most kMaxSegment: a wave walks a segment 8 entries at a time
// and the launch lasts as long as the longest walk, while the combine pass gives a row with many partial
// rows a whole workgroup (combine_kernel).
constexpr int64_t kMaxSegment = 24;      // measured: 24 beats 12, 16, 20, 32, 48 and 64 on the power-law and the headline workload
int32_t segment_len(int64_t k, const Options& opt) {
    int64_t s = std::min<int64_t>(kMaxSegment, (int64_t)std::ceil(std::sqrt((double)k)));
    return (int32_t)std::max<int64_t>(s, std::max(1, opt.min_segment));
}
}  // namespace

void make_pass_plan(int64_t n, const int32_t* ptr, const int32_t* idx_in, const Options& opt, PassPlan& out,
                    const uint32_t* flags_in, const uint32_t* row_bits, const uint8_t* skip) {
    // rows to leave out become empty rows of a CSR of their own, then one kSkipRow entry each, like split rows
    std::vector<int32_t> kept_ptr, kept_idx;
    std::vector<uint32_t> kept_flags;
    const int32_t* idx = idx_in;
    const uint32_t* flags = flags_in;
    if (skip) {
        kept_ptr.resize((size_t)n + 1);
        kept_ptr[0] = 0;
        for (int64_t r = 0; r < n; ++r) {
            if (!skip[(size_t)r])
                for (int32_t j = ptr[r]; j < ptr[r + 1]; ++j) {
                    kept_idx.push_back(idx_in[j]);
                    if (flags_in) kept_flags.push_back(flags_in[j]);
                }
            kept_ptr[(size_t)r + 1] = (int32_t)kept_idx.size();
        }
        ptr = kept_ptr.data();
        idx = kept_idx.data();
        if (flags_in) flags = kept_flags.data();
    }
    auto row_flag = [&](int64_t r) -> uint32_t { return row_bits && ((row_bits[(size_t)r >> 5] >> (r & 31)) & 1u) ? kRowFlag : 0u; };
    const int64_t e = ptr[n];
    out = PassPlan();
    if (flags)
        for (int64_t j = 0; j < e && !out.has_weighted; ++j) out.has_weighted = (flags[j] & kWeightedEdge) != 0;
    out.n_main = (int32_t)n;
    out.edges = e;
    int32_t heavy = std::max(1, opt.heavy_fan);
    {
        // A launch over the unsplit rows of a small pass lasts as long as its longest rows (a wave walks a row
        // 8 entries at a time).  Where rows are split anyway (so a lower threshold adds no launch), the unsplit
        // rows are few (the launch is bound by latency, not by what it moves) and rows longer than half the
        // threshold hold a tenth or more of their entries (power-law fan-ins), split from half the threshold on.
        // Measured at B = 64 on the two power-law workloads: 0.69 -> 0.64 ms and 0.75 -> 0.71 ms; the layered
        // workloads are 2-4% slower when every pass uses the lower threshold.
        const int32_t half = std::max(1, heavy / 2);
        int64_t light = 0, mid = 0;
        bool any_heavy = false;
        for (int64_t r = 0; r < n; ++r) {
            const int64_t k = ptr[r + 1] - ptr[r];
            if (k <= heavy) light += k;
            else any_heavy = true;
            if (k > half && k <= heavy) mid += k;
        }
        if (any_heavy && light < kLatencyBoundEntries && mid * 10 > light) heavy = half;
    }
    int64_t n_seg = 0, n_heavy = 0, heavy_edges = 0;
    for (int64_t r = 0; r < n; ++r) {
        int64_t k = ptr[r + 1] - ptr[r];
        if (k > heavy) {
            int32_t s = segment_len(k, opt);
            n_seg += (k + s - 1) / s;
            ++n_heavy;
            heavy_edges += k;
        }
    }
    out.n_seg = (int32_t)n_seg;
    out.n_heavy = (int32_t)n_heavy;
    out.ptr.resize((size_t)(n + n_seg + 1));
    int64_t n_skip = 0;
    if (skip)
        for (int64_t r = 0; r < n; ++r) n_skip += skip[(size_t)r] != 0;
    out.idx.assign((size_t)(e - heavy_edges + n_heavy + n_skip + heavy_edges + kIdxPad), 0u);
    out.seg_owner.resize((size_t)n_seg);
    out.comb_ptr.resize((size_t)(n_heavy + 1));
    out.comb_row.resize((size_t)n_heavy);
    // main rows keep their order and their entries come first; a split row is one kSkipRow entry
    int32_t w = 0;
    for (int64_t r = 0; r < n; ++r) {
        out.ptr[(size_t)r] = w;
        int64_t k = ptr[r + 1] - ptr[r];
        if (skip && skip[(size_t)r]) {
            out.idx[(size_t)w++] = kSkipRow;
        } else if (k <= heavy) {
            for (int64_t j = ptr[r]; j < ptr[r + 1]; ++j) out.idx[(size_t)w++] = (uint32_t)idx[j] | (flags ? flags[j] : 0u);
            if (k > 0) out.idx[(size_t)w - 1] |= kLastEdge | row_flag(r);
        } else {
            out.idx[(size_t)w++] = kSkipRow;
        }
    }
    out.ptr[(size_t)n] = w;
    // tasks: close a task once it holds `target` entries (or 64 rows)
    auto cut_tasks = [&](int64_t r_begin, int64_t r_end, std::vector<int32_t>& tasks) -> int32_t {
        const int64_t entries = out.ptr[(size_t)r_end] - out.ptr[(size_t)r_begin];
        const int64_t target = std::min<int64_t>(kTaskMax, std::max<int64_t>(kTaskMin, entries / kTaskDiv));
        tasks.clear();
        int64_t r = r_begin;
        while (r < r_end) {
            tasks.push_back((int32_t)r);
            tasks.push_back(out.ptr[(size_t)r]);
            int64_t r1 = r;
            while (r1 < r_end && r1 - r < 64 && out.ptr[(size_t)r1] - out.ptr[(size_t)r] < target) ++r1;
            r = r1;
        }
        const int32_t count = (int32_t)(tasks.size() / 2);
        tasks.push_back((int32_t)r_end);
        tasks.push_back(out.ptr[(size_t)r_end]);
        return count;
    };
    out.n_tasks = cut_tasks(0, n, out.tasks);
    if (n_heavy == 0) return;
    // Segments of all split rows, ordered by the first source they read: segments that read the
    // same stretch of source rows then run next to each other (and on the same XCD), so the
    // stretch is fetched once and served from L2 to the rest.
    struct Seg { int32_t owner, first_src; int64_t begin; int32_t len; };
    std::vector<Seg> segs;
    segs.reserve((size_t)n_seg);
    for (int64_t r = 0; r < n; ++r) {
        int64_t k = ptr[r + 1] - ptr[r];
        if (k <= heavy) continue;
        int32_t s = segment_len(k, opt);
        for (int64_t a = 0; a < k; a += s)
            segs.push_back(Seg{(int32_t)r, idx[ptr[r] + a], ptr[r] + a, (int32_t)std::min<int64_t>(s, k - a)});
    }
    std::stable_sort(segs.begin(), segs.end(), [](const Seg& a, const Seg& b) { return a.first_src < b.first_src; });
    // combine lists: scratch rows of each split row, in segment order
    std::vector<int32_t> per_owner_count((size_t)n, 0);
    for (const Seg& sg : segs) ++per_owner_count[(size_t)sg.owner];
    int64_t h = 0;
    std::vector<int32_t> owner_slot((size_t)n, -1);
    out.comb_ptr[0] = 0;
    for (int64_t r = 0; r < n; ++r)
        if (per_owner_count[(size_t)r] > 0) {
            owner_slot[(size_t)r] = (int32_t)h;
            out.comb_row[(size_t)h] = (int32_t)r;
            out.comb_ptr[(size_t)h + 1] = out.comb_ptr[(size_t)h] + per_owner_count[(size_t)r];
            ++h;
        }
    out.comb_idx.assign((size_t)n_seg + kIdxPad, 0u);
    std::vector<int32_t> fill(out.comb_ptr.begin(), out.comb_ptr.end() - 1);
    for (size_t sidx = 0; sidx < segs.size(); ++sidx) {
        const Seg& sg = segs[sidx];
        for (int64_t j = sg.begin; j < sg.begin + sg.len; ++j) out.idx[(size_t)w++] = (uint32_t)idx[j] | (flags ? flags[j] : 0u);
        out.idx[(size_t)w - 1] |= kLastEdge;
        out.seg_owner[sidx] = sg.owner;
        out.ptr[(size_t)n + sidx + 1] = w;
        out.comb_idx[(size_t)fill[(size_t)owner_slot[(size_t)sg.owner]]++] = (uint32_t)sidx;
    }
    for (int64_t hh = 0; hh < n_heavy; ++hh)
        out.comb_idx[(size_t)out.comb_ptr[(size_t)hh + 1] - 1] |= row_flag(out.comb_row[(size_t)hh]);
    out.n_seg_tasks = cut_tasks(n, n + n_seg, out.seg_tasks);
}

namespace {
// chunked, lane-interleaved index vectors of a CSR with n_src source rows, one run of lines per wave
// (see SlabPlan)
void make_slab(int64_t n, int64_t n_src, const int32_t* ptr, const int32_t* idx, const uint32_t* flags, SlabPlan& out,
               const uint32_t* row_bits = nullptr) {
    const int64_t chunks = (n + 63) / 64;
    std::vector<int32_t> width((size_t)chunks, 0);
    for (int64_t q = 0; q < chunks; ++q)
        for (int64_t r = q * 64; r < std::min<int64_t>(n, q * 64 + 64); ++r)
            width[(size_t)q] = std::max(width[(size_t)q], ptr[r + 1] - ptr[r]);
    for (int32_t& w : width) w = std::max(w, 1);      // every chunk has a last line, also one of empty rows
    int64_t lines = 0;
    for (int w = 0; w < kSlabWaves; ++w) {
        out.wave_line[w] = (int32_t)lines;
        for (int64_t q = w; q < chunks; q += kSlabWaves) lines += width[(size_t)q];
        lines = (lines + kSlabBlock - 1) / kSlabBlock * kSlabBlock;
    }
    out.wave_line[kSlabWaves] = (int32_t)lines;
    out.ent.assign((size_t)lines * 64, (uint32_t)n_src);
    for (int w = 0; w < kSlabWaves; ++w) {
        int64_t line = out.wave_line[w];
        for (int64_t q = w; q < chunks; q += kSlabWaves) {
            const int32_t wq = width[(size_t)q];
            for (int64_t r = q * 64; r < std::min<int64_t>(n, q * 64 + 64); ++r)
                for (int32_t j = ptr[r]; j < ptr[r + 1]; ++j)
                    out.ent[(size_t)(line + (j - ptr[r])) * 64 + (size_t)(r - q * 64)] = (uint32_t)idx[j] | (flags ? flags[j] : 0u);
            for (int lane = 0; lane < 64; ++lane) {
                uint32_t& last = out.ent[(size_t)(line + wq - 1) * 64 + (size_t)lane];
                last |= kLastEdge;
                // the word a lane holds when its chunk closes also tells whether its row is flagged
                const int64_t r = q * 64 + lane;
                if (row_bits && r < n && ((row_bits[(size_t)r >> 5] >> (r & 31)) & 1u)) last |= kRowFlag;
            }
            line += wq;
        }
    }
}
}  // namespace

int layerize(int32_t V, int64_t N, const uint8_t* node_type, const int32_t* node_lit,
             const int64_t* child_ptr, const int32_t* child_idx_in, int32_t R, const int32_t* roots_in,
             const Options& opt, CircuitPlan& plan, std::string& err) {
    plan = CircuitPlan();
    const int32_t* child_idx = child_idx_in;
    const int32_t* roots = roots_in;
    // ---------------------------------------------------------------- validation
    if (V < 0 || N <= 0 || R <= 0 || !node_type || !node_lit || !child_ptr || !roots) {
        err = "klay_build: null array or non-positive size";
        return ST_INVAL;
    }
    if (N >= INT32_MAX) { err = "klay_build: more than 2^31-1 nodes"; return ST_INVAL; }
    if (child_ptr[0] != 0) { err = "klay_build: child_ptr[0] must be 0"; return ST_INVAL; }
    for (int64_t i = 0; i < N; ++i)
        if (child_ptr[i + 1] < child_ptr[i]) { err = "klay_build: child_ptr is not monotone"; return ST_INVAL; }
    const int64_t E = child_ptr[N];
    if (E > 0 && !child_idx) { err = "klay_build: child_idx is null"; return ST_INVAL; }
    for (int64_t i = 0; i < N; ++i) {
        const int64_t k = child_ptr[i + 1] - child_ptr[i];
        switch (node_type[i]) {
        case T_LIT: {
            int64_t l = node_lit[i];
            if (l == 0 || std::llabs(l) > V) {
                err = "klay_build: literal of node " + std::to_string(i) + " out of range";
                return ST_INVAL;
            }
        }   // fallthrough
        case T_TRUE:
        case T_FALSE:
            if (k != 0) { err = "klay_build: leaf node " + std::to_string(i) + " has children"; return ST_INVAL; }
            break;
        case T_AND:
        case T_OR:
            if (k == 0) { err = "klay_build: gate " + std::to_string(i) + " has no children"; return ST_INVAL; }
            break;
        default:
            err = "klay_build: unknown node type at node " + std::to_string(i);
            return ST_INVAL;
        }
    }
    for (int64_t j = 0; j < E; ++j)
        if (child_idx[j] < 0 || child_idx[j] >= N) { err = "klay_build: child index out of range"; return ST_INVAL; }
    for (int32_t r = 0; r < R; ++r)
        if (roots[r] < 0 || roots[r] >= N) { err = "klay_build: root index out of range"; return ST_INVAL; }

    // Leaves that carry the same literal (or the same constant) are one node: every reference is
    // redirected to the first of them (the leaf case of the node identification of Section 3.2).
    std::vector<int32_t> cidx((size_t)E), croots((size_t)R);
    {
        std::vector<int32_t> first_lit((size_t)2 * V + 2, -1), canon((size_t)N);
        for (int64_t i = 0; i < N; ++i) {
            canon[(size_t)i] = (int32_t)i;
            int64_t slot = -1;
            if (node_type[i] == T_LIT) slot = 2 * (std::llabs((int64_t)node_lit[i]) - 1) + (node_lit[i] < 0 ? 1 : 0);
            else if (node_type[i] == T_TRUE) slot = 2 * (int64_t)V;
            else if (node_type[i] == T_FALSE) slot = 2 * (int64_t)V + 1;
            if (slot >= 0) {
                if (first_lit[(size_t)slot] < 0) first_lit[(size_t)slot] = (int32_t)i;
                canon[(size_t)i] = first_lit[(size_t)slot];
            }
        }
        for (int64_t j = 0; j < E; ++j) cidx[(size_t)j] = canon[(size_t)child_idx[j]];
        for (int32_t r = 0; r < R; ++r) croots[(size_t)r] = canon[(size_t)roots[r]];
        child_idx = cidx.data();
        roots = croots.data();
    }

    // ---------------------------------------------------------------- parents of every node
    std::vector<int64_t> par_ptr((size_t)N + 1, 0);
    for (int64_t j = 0; j < E; ++j) ++par_ptr[(size_t)child_idx[j] + 1];
    for (int64_t i = 0; i < N; ++i) par_ptr[(size_t)i + 1] += par_ptr[(size_t)i];
    std::vector<int32_t> par_idx((size_t)E);
    {
        std::vector<int64_t> fill(par_ptr.begin(), par_ptr.end() - 1);
        for (int64_t i = 0; i < N; ++i)
            for (int64_t j = child_ptr[i]; j < child_ptr[i + 1]; ++j) par_idx[(size_t)fill[(size_t)child_idx[j]]++] = (int32_t)i;
    }

    // ---------------------------------------------------------------- heights, children first (Eq. 2)
    // h = 0 for leaves, 1 + max over children otherwise; a gate whose parity disagrees with its
    // type (AND must sit on an odd layer, OR on an even one) is lifted by one layer.
    std::vector<int32_t> h((size_t)N, 0);
    std::vector<int32_t> topo;                  // every node, children before parents
    topo.reserve((size_t)N);
    {
        std::vector<int64_t> pending((size_t)N);
        std::vector<int32_t> ready;
        ready.reserve((size_t)N);
        for (int64_t i = 0; i < N; ++i) {
            pending[(size_t)i] = child_ptr[i + 1] - child_ptr[i];
            if (pending[(size_t)i] == 0) ready.push_back((int32_t)i);
        }
        int64_t done = 0;
        while (!ready.empty()) {
            int32_t n = ready.back();
            ready.pop_back();
            ++done;
            topo.push_back(n);
            if (node_type[n] == T_AND || node_type[n] == T_OR) {
                int32_t m = 0;
                for (int64_t j = child_ptr[n]; j < child_ptr[n + 1]; ++j) m = std::max(m, h[(size_t)child_idx[j]]);
                int32_t hn = m + 1;
                const bool odd = (hn & 1) != 0;
                if ((node_type[n] == T_AND) != odd) ++hn;
                h[(size_t)n] = hn;
            }
            for (int64_t j = par_ptr[(size_t)n]; j < par_ptr[(size_t)n + 1]; ++j)
                if (--pending[(size_t)par_idx[(size_t)j]] == 0) ready.push_back(par_idx[(size_t)j]);
        }
        if (done != N) { err = "klay_build: the node graph has a cycle"; return ST_CYCLE; }
    }

    // ---------------------------------------------------------------- identical sub-circuits (Section 3.2, Eq. 3, Theorem 1)
    // Bottom-up, a gate is identified by its type and the multiset of its (already identified)
    // children.  The hash is a permutation-invariant sum of mixed child ids; on a hash hit the child
    // lists are compared, so a collision can never merge different gates.  Identical gates have
    // identical heights, so the layers computed above stay valid.
    if (!opt.no_merge) {
        auto mix = [](uint64_t x) {
            x += 0x9E3779B97F4A7C15ull;
            x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
            x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
            return x ^ (x >> 31);
        };
        std::vector<int32_t> rep((size_t)N);
        std::iota(rep.begin(), rep.end(), 0);
        std::unordered_map<uint64_t, int32_t> head;
        head.reserve((size_t)N);
        std::vector<int32_t> next_same((size_t)N, -1);
        for (int32_t n : topo) {
            if (node_type[n] != T_AND && node_type[n] != T_OR) continue;
            const int64_t a = child_ptr[n], b = child_ptr[n + 1];
            for (int64_t j = a; j < b; ++j) cidx[(size_t)j] = rep[(size_t)cidx[(size_t)j]];
            std::sort(cidx.begin() + a, cidx.begin() + b);
            uint64_t hsh = mix((uint64_t)node_type[n] * 0x51ED27ull + (uint64_t)(b - a));
            for (int64_t j = a; j < b; ++j) hsh += mix((uint64_t)cidx[(size_t)j]);
            auto it = head.find(hsh);
            int32_t found = -1;
            if (it != head.end()) {
                for (int32_t m = it->second; m >= 0; m = next_same[(size_t)m]) {
                    const int64_t ma = child_ptr[m], mb = child_ptr[m + 1];
                    if (node_type[m] == node_type[n] && mb - ma == b - a &&
                        std::equal(cidx.begin() + a, cidx.begin() + b, cidx.begin() + ma)) { found = m; break; }
                }
            }
            if (found >= 0) {
                rep[(size_t)n] = found;
                ++plan.num_merged;
            } else if (it != head.end()) {
                next_same[(size_t)n] = it->second;
                it->second = n;
            } else {
                head.emplace(hsh, n);
            }
        }
        for (int32_t r = 0; r < R; ++r) croots[(size_t)r] = rep[(size_t)croots[(size_t)r]];
    }

    // ---------------------------------------------------------------- reachability from the roots
    std::vector<uint8_t> reach((size_t)N, 0);
    {
        std::vector<int32_t> stack;
        for (int32_t r = 0; r < R; ++r)
            if (!reach[(size_t)roots[r]]) { reach[(size_t)roots[r]] = 1; stack.push_back(roots[r]); }
        while (!stack.empty()) {
            int32_t n = stack.back();
            stack.pop_back();
            for (int64_t j = child_ptr[n]; j < child_ptr[n + 1]; ++j) {
                int32_t c = child_idx[j];
                if (!reach[(size_t)c]) { reach[(size_t)c] = 1; stack.push_back(c); }
            }
        }
    }
    // A gate that is part of the circuit must not name the same input node twice (the children of a
    // gate are a set, Eq. 1).  Checked on the ids as given: two different leaf nodes that carry the same
    // literal, or two gates that turn out identical, are two children and count twice, as in Eq. 1.
    {
        std::vector<int32_t> stamp((size_t)N, -1);
        for (int64_t i = 0; i < N; ++i) {
            if (!reach[(size_t)i]) continue;
            for (int64_t j = child_ptr[i]; j < child_ptr[i + 1]; ++j) {
                const int32_t c = child_idx_in[j];
                if (stamp[(size_t)c] == (int32_t)i) { err = "klay_build: gate " + std::to_string(i) + " lists a child twice"; return ST_INVAL; }
                stamp[(size_t)c] = (int32_t)i;
            }
        }
    }
    int32_t L = 0;
    for (int32_t r = 0; r < R; ++r) L = std::max(L, h[(size_t)roots[r]]);

    // ---------------------------------------------------------------- unary chains (Section 3.1; one per (child, layer))
    // need[c] = highest layer at which a stand-in for c is read: parent height - 1, or L for roots.
    std::vector<int32_t> need(h);
    std::vector<int32_t> max_fan((size_t)L + 1, 0);       // largest fan-in among the gates of a layer
    for (int64_t p = 0; p < N; ++p) {
        if (!reach[(size_t)p]) continue;
        plan.dag_nodes++;
        plan.dag_edges += child_ptr[p + 1] - child_ptr[p];
        max_fan[(size_t)h[(size_t)p]] = (int32_t)std::max<int64_t>(max_fan[(size_t)h[(size_t)p]], child_ptr[p + 1] - child_ptr[p]);
        for (int64_t j = child_ptr[p]; j < child_ptr[p + 1]; ++j) {
            int32_t c = child_idx[j];
            need[(size_t)c] = std::max(need[(size_t)c], h[(size_t)p] - 1);
        }
    }
    for (int32_t r = 0; r < R; ++r) need[(size_t)roots[r]] = L;

    // Padding-free lower part (Options::alias_chains): the layers 1 .. B0 (B0 = plan.alias_top) hold no
    // stand-ins except that layer B0 is complete: it holds a stand-in for every node that a layer above
    // reads.  The edges of the layers up to B0 name the child's own row in the whole activation buffer,
    // wherever it lives; from layer B0 + 1 on every edge goes to the layer directly below, as in the
    // paper.  B0 is chosen so that the layers above it are exactly the narrow top of the circuit that the
    // persistent kernels can take (they need complete layers); B0 = 0 is the paper's layerization, B0 = L
    // has no chain nodes at all except the stand-ins that bring every root to the top layer.
    const int64_t rows_cap = opt.tail_rows_cap > 0 ? std::min<int64_t>(opt.tail_rows_cap, kTailRowsCap) : kTailRowsCap;
    int32_t B0 = 0;
    {
        std::vector<int64_t> full((size_t)L + 1, 0);       // layer sizes with all chain nodes
        for (int64_t c = 0; c < N; ++c)
            if (reach[(size_t)c])
                for (int32_t l = h[(size_t)c]; l <= need[(size_t)c]; ++l) ++full[(size_t)l];
        if (opt.alias_chains) {
            B0 = L;
            if (!opt.no_tail) {
                int32_t t = L + 1;
                while (t - 1 >= 1 && full[(size_t)t - 1] <= rows_cap && full[(size_t)t - 2] <= rows_cap &&
                       max_fan[(size_t)t - 1] <= kTailFanCap)
                    --t;
                if (L - t + 1 >= 2) B0 = t - 1;            // a persistent kernel takes two layers or more
            }
        }
    }
    plan.alias_top = B0;
    plan.alias = B0 > 0;
    // lowest level at which c has a stand-in (none if that is above need[c])
    auto lo = [&](int64_t c) { return std::max(h[(size_t)c] + 1, B0); };

    // Fused AND rows (see LayerPlan): AND nodes of the padding-free part whose value nothing has to read.
    std::vector<uint8_t> fused((size_t)N, 0);
    if (B0 > 0 && !opt.no_fusion) {
        // a row is split when it has more entries than heavy_fan, or than half of it (make_pass_plan): the rows that
        // read through fused rows stay at or below that, so that no group of entries is cut by a segment boundary
        const int64_t row_max = std::min<int64_t>(kFusedRowMax, std::max(1, opt.heavy_fan / 2));
        std::vector<uint8_t> cand((size_t)N, 0);
        for (int64_t c = 0; c < N; ++c) {
            if (!reach[(size_t)c] || !(h[(size_t)c] & 1) || h[(size_t)c] >= B0 || need[(size_t)c] >= B0) continue;
            const int64_t fi = child_ptr[c + 1] - child_ptr[c];
            int64_t gates = 0;
            for (int64_t j = child_ptr[c]; j < child_ptr[c + 1]; ++j) gates += h[(size_t)child_idx[j]] > 0;
            cand[(size_t)c] = fi >= 1 && gates <= 1 && fi <= row_max;
        }
        // every parent has to be an OR row that stays short when it reads the children of its fused children
        for (int64_t p = 0; p < N; ++p) {
            if (!reach[(size_t)p] || h[(size_t)p] == 0) continue;
            int64_t len = 0;
            bool any = false;
            for (int64_t j = child_ptr[p]; j < child_ptr[p + 1]; ++j) {
                const int32_t c = child_idx[j];
                any = any || (cand[(size_t)c] & 1);
                len += (cand[(size_t)c] & 1) ? child_ptr[c + 1] - child_ptr[c] : 1;
            }
            if (!any || ((h[(size_t)p] & 1) == 0 && len <= row_max)) continue;
            for (int64_t j = child_ptr[p]; j < child_ptr[p + 1]; ++j) cand[(size_t)child_idx[j]] |= 2;      // not through this parent
        }
        for (int64_t c = 0; c < N; ++c)
            if (cand[(size_t)c] == 1) { fused[(size_t)c] = 1; ++plan.num_fused; }
    }

    std::vector<int64_t> count((size_t)L + 1, 0);
    std::vector<int64_t> pad_base((size_t)N + 1, 0);
    for (int64_t c = 0; c < N; ++c) {
        pad_base[(size_t)c + 1] = pad_base[(size_t)c];
        if (!reach[(size_t)c]) continue;
        ++count[(size_t)h[(size_t)c]];
        const int32_t pads = std::max(0, need[(size_t)c] - lo(c) + 1);
        pad_base[(size_t)c + 1] += pads;
        for (int32_t l = lo(c); l <= need[(size_t)c]; ++l) ++count[(size_t)l];
    }
    plan.num_pad_nodes = pad_base[(size_t)N];
    for (int32_t l = 0; l <= L; ++l)
        if (count[(size_t)l] >= INT32_MAX) { err = "klay_build: a layer has more than 2^31-1 nodes"; return ST_INVAL; }

    // slot of every node within its layer before ordering: real nodes by id, then chain nodes by id
    std::vector<int32_t> pos_real((size_t)N, -1);
    std::vector<int32_t> pos_pad((size_t)plan.num_pad_nodes, -1);
    plan.layers.resize((size_t)L + 1);
    {
        std::vector<int64_t> fill((size_t)L + 1, 0);
        for (int32_t l = 0; l <= L; ++l) {
            plan.layers[(size_t)l].n = count[(size_t)l];
            plan.layers[(size_t)l].origin.resize((size_t)count[(size_t)l]);
            plan.layers[(size_t)l].is_pad.assign((size_t)count[(size_t)l], 0);
        }
        for (int64_t c = 0; c < N; ++c)
            if (reach[(size_t)c]) {
                int32_t l = h[(size_t)c];
                pos_real[(size_t)c] = (int32_t)fill[(size_t)l];
                plan.layers[(size_t)l].origin[(size_t)fill[(size_t)l]++] = (int32_t)c;
            }
        for (int64_t c = 0; c < N; ++c)
            if (reach[(size_t)c])
                for (int32_t l = lo(c); l <= need[(size_t)c]; ++l) {
                    pos_pad[(size_t)(pad_base[(size_t)c] + l - lo(c))] = (int32_t)fill[(size_t)l];
                    plan.layers[(size_t)l].origin[(size_t)fill[(size_t)l]] = (int32_t)c;
                    plan.layers[(size_t)l].is_pad[(size_t)fill[(size_t)l]++] = 1;
                }
    }
    plan.row0.assign((size_t)L + 2, 0);
    for (int32_t l = 0; l <= L; ++l) plan.row0[(size_t)l + 1] = plan.row0[(size_t)l] + count[(size_t)l];
    if (plan.row0[(size_t)L + 1] + R >= kMaxRows) { err = "klay_build: more than 2^29 rows"; return ST_INVAL; }
    // position, within layer `level`, of node c or of its stand-in there (c is present at that level)
    auto at = [&](int32_t c, int32_t level) -> int32_t {
        return level == h[(size_t)c] ? pos_real[(size_t)c] : pos_pad[(size_t)(pad_base[(size_t)c] + level - lo(c))];
    };
    // what an edge from layer level + 1 down to c holds: below B0 the row of c itself in the whole
    // activation buffer, from B0 on the position of c (or of its stand-in) in layer `level`
    auto src_at = [&](int32_t c, int32_t level) -> int32_t {
        if (level < B0) return (int32_t)(plan.row0[(size_t)h[(size_t)c]] + pos_real[(size_t)c]);
        return at(c, level);
    };
    // ordering key of a child: its position in the layer below, or (below the boundary layer) its relative
    // position within its own layer scaled to the width of the layer below
    auto child_key = [&](int32_t c, int32_t level) -> double {
        if (level >= B0) return (double)at(c, level);
        const int32_t hc = h[(size_t)c];
        return (double)pos_real[(size_t)c] / (double)std::max<int64_t>(1, count[(size_t)hc]) * (double)count[(size_t)level];
    };
    auto set_at = [&](int32_t c, int32_t level, int32_t p) {
        if (level == h[(size_t)c]) pos_real[(size_t)c] = p;
        else pos_pad[(size_t)(pad_base[(size_t)c] + level - lo(c))] = p;
    };

    // ---------------------------------------------------------------- node order within layers (Section 4: arbitrary)
    // Layer 0: by variable, positive literal first, then constants.  Higher layers: by the smallest
    // position among a node's children in the layer below (one bottom-up sweep; ties keep slot
    // order): every row of the layer below is then first read in storage order, a sequential
    // stream, and only the remaining reads of a row are scattered.  (Measured on the headline
    // circuit: 12% faster than input order, 2% faster than ordering by the mean child position.)
    // AND layers are then re-ordered by their first parent (see below).
    auto apply_order = [&](int32_t l, const std::vector<int32_t>& order /* new position -> old slot */) {
        LayerPlan& lay = plan.layers[(size_t)l];
        std::vector<int32_t> origin(lay.origin.size());
        std::vector<uint8_t> is_pad(lay.is_pad.size());
        for (size_t p = 0; p < order.size(); ++p) {
            origin[p] = lay.origin[(size_t)order[p]];
            is_pad[p] = lay.is_pad[(size_t)order[p]];
            set_at(origin[p], l, (int32_t)p);
        }
        lay.origin.swap(origin);
        lay.is_pad.swap(is_pad);
    };
    {
        LayerPlan& l0 = plan.layers[0];
        std::vector<int32_t> order((size_t)l0.n);
        std::iota(order.begin(), order.end(), 0);
        auto key = [&](int32_t slot) -> int64_t {
            int32_t c = l0.origin[(size_t)slot];
            if (node_type[c] == T_LIT) {
                int64_t lit = node_lit[c];
                return 2 * (std::llabs(lit) - 1) + (lit < 0 ? 1 : 0);
            }
            return 2 * (int64_t)V + (node_type[c] == T_TRUE ? 0 : 1);
        };
        std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return key(a) < key(b); });
        apply_order(0, order);
    }
    if (!opt.no_reorder) {
        auto order_by_children = [&](int32_t l) {
            LayerPlan& lay = plan.layers[(size_t)l];
            std::vector<double> key((size_t)lay.n);
            for (int64_t s = 0; s < lay.n; ++s) {
                int32_t c = lay.origin[(size_t)s];
                if (lay.is_pad[(size_t)s]) key[(size_t)s] = child_key(c, l - 1);
                else {
                    double acc = 1e300;
                    for (int64_t j = child_ptr[c]; j < child_ptr[c + 1]; ++j) acc = std::min(acc, child_key(child_idx[j], l - 1));
                    key[(size_t)s] = acc;
                }
            }
            std::vector<int32_t> order((size_t)lay.n);
            std::iota(order.begin(), order.end(), 0);
            std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return key[(size_t)a] < key[(size_t)b]; });
            if (lay.n <= rows_cap && l >= B0 && !opt.no_tail) {
                // A layer small enough for the persistent top-of-circuit kernels: there a thread walks a whole
                // row and a wave waits for its longest one, while locality is irrelevant (the layer sits in
                // LDS).  Group rows by fan-in (powers of two) and order each group by fan-out, so that the 64
                // rows of a wave have similar lengths in the forward and in the reverse sweep.
                std::vector<int32_t> fan_in((size_t)lay.n), fan_out((size_t)lay.n, 0);
                for (int64_t s2 = 0; s2 < lay.n; ++s2) {
                    const int32_t c = lay.origin[(size_t)s2];
                    fan_in[(size_t)s2] = lay.is_pad[(size_t)s2] ? 1 : (int32_t)(child_ptr[c + 1] - child_ptr[c]);
                }
                if (l < L) {
                    const LayerPlan& up = plan.layers[(size_t)l + 1];
                    for (int64_t s2 = 0; s2 < up.n; ++s2) {
                        const int32_t c = up.origin[(size_t)s2];
                        if (up.is_pad[(size_t)s2]) ++fan_out[(size_t)at(c, l)];
                        else
                            for (int64_t j = child_ptr[c]; j < child_ptr[c + 1]; ++j) ++fan_out[(size_t)at(child_idx[j], l)];
                    }
                }
                auto bucket = [](int32_t k) { int b = 0; while ((1 << b) < k) ++b; return b; };
                std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
                    const int ba = bucket(fan_in[(size_t)a]), bb = bucket(fan_in[(size_t)b]);
                    if (ba != bb) return ba > bb;
                    return fan_out[(size_t)a] > fan_out[(size_t)b];
                });
            }
            apply_order(l, order);
        };
        for (int32_t l = 1; l <= L; ++l) order_by_children(l);
        // Second sweep, from the top, over the AND layers only: a row moves next to the first of its
        // parents, so the children of an OR node sit together.  The reverse sweep of an OR layer reads two
        // rows per edge (adjoint and value of the parent) against one in every other pass, so that pass
        // gets the locality: its gathers of a parent's rows then hit in L2 for the siblings.  (Measured on
        // the headline circuit: 2.4% of the step; doing the same for the OR layers, or iterating the two
        // sweeps, gains nothing more.)
        auto order_by_parents = [&](int32_t l) {
            LayerPlan& lay = plan.layers[(size_t)l];
            if (lay.n <= rows_cap && !opt.no_tail) return;       // keep the fan-sorted order of small layers
            const LayerPlan& up = plan.layers[(size_t)l + 1];
            std::vector<int32_t> key((size_t)lay.n, INT32_MAX);
            for (int64_t p2 = 0; p2 < up.n; ++p2) {
                const int32_t c = up.origin[(size_t)p2];
                if (up.is_pad[(size_t)p2]) { int32_t& k2 = key[(size_t)at(c, l)]; k2 = std::min<int32_t>(k2, (int32_t)p2); }
                else
                    for (int64_t j = child_ptr[c]; j < child_ptr[c + 1]; ++j) {
                        int32_t& k2 = key[(size_t)at(child_idx[j], l)];
                        k2 = std::min<int32_t>(k2, (int32_t)p2);
                    }
            }
            std::vector<int32_t> order((size_t)lay.n);
            std::iota(order.begin(), order.end(), 0);
            std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return key[(size_t)a] < key[(size_t)b]; });
            apply_order(l, order);
        };
        // (layers from B0 on: their parents sit in the layer directly above)
        for (int32_t l = L - 1; l >= std::max(B0, 1); --l)
            if (l & 1) order_by_parents(l);
        if (B0 > 0) {
            // the same idea for the layers below B0, whose parents sit in any higher layer up to B0: one sweep
            // from the top keeps, per node, the smallest relative position among its parents seen so far
            std::vector<double> pkey((size_t)N, 2.0);
            for (int32_t l = B0; l >= 1; --l) {
                LayerPlan& lay = plan.layers[(size_t)l];
                if ((l & 1) && l < B0) {
                    std::vector<int32_t> order((size_t)lay.n);
                    std::iota(order.begin(), order.end(), 0);
                    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
                        return pkey[(size_t)lay.origin[(size_t)a]] < pkey[(size_t)lay.origin[(size_t)b]];
                    });
                    apply_order(l, order);
                }
                for (int64_t s2 = 0; s2 < lay.n; ++s2) {
                    const int32_t c = lay.origin[(size_t)s2];
                    const double rel = ((double)s2 + 0.5) / (double)lay.n;
                    if (lay.is_pad[(size_t)s2]) { pkey[(size_t)c] = std::min(pkey[(size_t)c], rel); continue; }
                    for (int64_t j = child_ptr[c]; j < child_ptr[c + 1]; ++j) pkey[(size_t)child_idx[j]] = std::min(pkey[(size_t)child_idx[j]], rel);
                }
            }
        }
    }

    // the row of node x in the whole activation buffer (the padding-free part)
    auto own_row = [&](int32_t x) -> int32_t { return (int32_t)(plan.row0[(size_t)h[(size_t)x]] + pos_real[(size_t)x]); };

    // ---------------------------------------------------------------- index vectors per layer (Alg. 3), CSR by parent
    Options popt = opt;
    for (int32_t l = 1; l <= L; ++l) {
        LayerPlan& lay = plan.layers[(size_t)l];
        int64_t e = 0;
        for (int64_t p = 0; p < lay.n; ++p)
            e += lay.is_pad[(size_t)p] ? 1 : child_ptr[lay.origin[(size_t)p] + 1] - child_ptr[lay.origin[(size_t)p]];
        if (e + lay.n >= INT32_MAX - 64) { err = "klay_build: a layer has more than 2^31 edges"; return ST_INVAL; }
        lay.e = e;
        lay.row_ptr.resize((size_t)lay.n + 1);
        lay.child.resize((size_t)e);
        int32_t w = 0;
        for (int64_t p = 0; p < lay.n; ++p) {
            lay.row_ptr[(size_t)p] = w;
            int32_t c = lay.origin[(size_t)p];
            if (lay.is_pad[(size_t)p]) lay.child[(size_t)w++] = src_at(c, l - 1);
            else {
                const int32_t w0 = w;
                for (int64_t j = child_ptr[c]; j < child_ptr[c + 1]; ++j) lay.child[(size_t)w++] = src_at(child_idx[j], l - 1);
                std::sort(lay.child.begin() + w0, lay.child.begin() + w);
            }
            plan.max_fan_in = std::max<int64_t>(plan.max_fan_in, w - lay.row_ptr[(size_t)p]);
        }
        lay.row_ptr[(size_t)lay.n] = w;
        lay.multi.assign((size_t)(lay.n + 31) / 32, 0u);
        for (int64_t p = 0; p < lay.n; ++p)
            if (lay.row_ptr[(size_t)p + 1] - lay.row_ptr[(size_t)p] > 1) lay.multi[(size_t)p >> 5] |= 1u << (p & 31);
        make_pass_plan(lay.n, lay.row_ptr.data(), lay.child.data(), popt, lay.fwd);
        if ((l & 1) && l < B0 && plan.num_fused > 0) {
            std::vector<uint8_t> skip((size_t)lay.n, 0);
            for (int64_t p = 0; p < lay.n; ++p) {
                skip[(size_t)p] = fused[(size_t)lay.origin[(size_t)p]];
                lay.n_fused += skip[(size_t)p];
            }
            if (lay.n_fused > 0 && lay.n_fused < lay.n)
                make_pass_plan(lay.n, lay.row_ptr.data(), lay.child.data(), popt, lay.fwd_kept, nullptr, nullptr, skip.data());
        }
        if ((l & 1) == 0 && l <= B0 && plan.num_fused > 0) {
            // fwd2: every child of an OR row as a group of entries; a fused AND child is replaced by its children
            bool reads_fused = false;
            std::vector<int32_t> ptr2((size_t)lay.n + 1, 0), idx2;
            std::vector<uint32_t> flag2;
            idx2.reserve((size_t)e * 2);
            flag2.reserve((size_t)e * 2);
            std::vector<std::pair<int32_t, int32_t>> kids;       // (row, node) of a row's children, by row
            std::vector<int32_t> grp;
            for (int64_t p = 0; p < lay.n; ++p) {
                const int32_t c = lay.origin[(size_t)p];
                if (lay.is_pad[(size_t)p]) {
                    idx2.push_back(lay.child[(size_t)lay.row_ptr[(size_t)p]]);
                    flag2.push_back(kGroupEnd);
                } else {
                    kids.clear();
                    for (int64_t j = child_ptr[c]; j < child_ptr[c + 1]; ++j) kids.emplace_back(own_row(child_idx[j]), child_idx[j]);
                    std::sort(kids.begin(), kids.end());
                    for (const auto& kid : kids) {
                        if (!fused[(size_t)kid.second]) {
                            idx2.push_back(kid.first);
                            flag2.push_back(kGroupEnd);
                            continue;
                        }
                        reads_fused = true;
                        const int32_t a = kid.second;
                        grp.clear();
                        for (int64_t j = child_ptr[a]; j < child_ptr[a + 1]; ++j) grp.push_back(own_row(child_idx[j]));
                        std::sort(grp.begin(), grp.end());
                        for (size_t g = 0; g < grp.size(); ++g) {
                            idx2.push_back(grp[g]);
                            flag2.push_back(g + 1 == grp.size() ? kGroupEnd : 0u);
                        }
                    }
                }
                if (idx2.size() >= (size_t)INT32_MAX - 64) { err = "klay_build: a layer has more than 2^31 edges"; return ST_INVAL; }
                ptr2[(size_t)p + 1] = (int32_t)idx2.size();
            }
            if (reads_fused) {
                make_pass_plan(lay.n, ptr2.data(), idx2.data(), popt, lay.fwd2, flag2.data());
                plan.max_fwd_seg = std::max<int64_t>(plan.max_fwd_seg, lay.fwd2.n_seg);
            }
        }

        plan.num_edges += e;
        plan.num_split_rows += lay.fwd.n_heavy;
        plan.max_fwd_seg = std::max<int64_t>(plan.max_fwd_seg, lay.fwd.n_seg);
        if (l <= B0) continue;             // their reverse plans are built below, over the whole lower part

        // by child (for the reverse sweep): rows = nodes of layer l-1, sources = parents in layer l;
        // an edge is weighted when its parent is an OR node with more than one child
        const int64_t nc = plan.layers[(size_t)l - 1].n;
        std::vector<int32_t> cptr((size_t)nc + 1, 0), cpar((size_t)e);
        std::vector<uint32_t> cflag((size_t)e, 0u);
        for (int64_t j = 0; j < e; ++j) ++cptr[(size_t)lay.child[(size_t)j] + 1];
        for (int64_t i = 0; i < nc; ++i) {
            plan.max_fan_out = std::max<int64_t>(plan.max_fan_out, cptr[(size_t)i + 1]);
            cptr[(size_t)i + 1] += cptr[(size_t)i];
        }
        {
            std::vector<int32_t> fill(cptr.begin(), cptr.end() - 1);
            for (int64_t p = 0; p < lay.n; ++p)
                for (int32_t j = lay.row_ptr[(size_t)p]; j < lay.row_ptr[(size_t)p + 1]; ++j) {
                    const int32_t slot = fill[(size_t)lay.child[(size_t)j]]++;
                    cpar[(size_t)slot] = (int32_t)p;
                    if ((l & 1) == 0 && lay.row_ptr[(size_t)p + 1] - lay.row_ptr[(size_t)p] > 1) cflag[(size_t)slot] = kWeightedEdge;
                }
        }
        // the rows of this pass are the nodes of layer l - 1: below an AND layer they are OR nodes, and those
        // with more than one child are flagged (their adjoints are stored in the one-gather form)
        make_pass_plan(nc, cptr.data(), cpar.data(), popt, lay.bwd, cflag.data(),
                       (l & 1) && l >= 3 ? plan.layers[(size_t)l - 1].multi.data() : nullptr);
        if (!opt.no_tail && lay.n <= rows_cap && nc <= rows_cap) {
            int64_t fan_in = 0, fan_out = 0;
            for (int64_t i = 0; i < lay.n; ++i) fan_in = std::max<int64_t>(fan_in, lay.row_ptr[(size_t)i + 1] - lay.row_ptr[(size_t)i]);
            for (int64_t i = 0; i < nc; ++i) fan_out = std::max<int64_t>(fan_out, cptr[(size_t)i + 1] - cptr[(size_t)i]);
            if (fan_in <= kTailFanCap) {
                make_slab(lay.n, nc, lay.row_ptr.data(), lay.child.data(), nullptr, lay.slab_fwd);
                lay.tail_fwd_ok = true;
                if (fan_out <= kTailFanCap) {
                    make_slab(nc, lay.n, cptr.data(), cpar.data(), cflag.data(), lay.slab_bwd,
                              (l & 1) && l >= 3 ? plan.layers[(size_t)l - 1].multi.data() : nullptr);
                    lay.tail_bwd_ok = true;
                }
            }
        }
        plan.num_split_rows += lay.bwd.n_heavy;
        plan.max_bwd_seg = std::max<int64_t>(plan.max_bwd_seg, lay.bwd.n_seg);
    }
    if (B0 > 0) {
        // Reverse-sweep sources of every row below layer B0: its parents, which are rows of any higher
        // layer up to B0 (adjoint rows are numbered like the rows of the activation buffer).
        const int64_t NR = plan.row0[(size_t)B0];
        std::vector<int32_t> gptr((size_t)NR + 1, 0);
        for (int32_t l = 1; l <= B0; ++l)
            for (int32_t ch : plan.layers[(size_t)l].child) ++gptr[(size_t)ch + 1];
        for (int64_t i = 0; i < NR; ++i) {
            plan.max_fan_out = std::max<int64_t>(plan.max_fan_out, gptr[(size_t)i + 1]);
            if ((int64_t)gptr[(size_t)i] + gptr[(size_t)i + 1] >= INT32_MAX - 64) { err = "klay_build: more than 2^31 edges"; return ST_INVAL; }
            gptr[(size_t)i + 1] += gptr[(size_t)i];
        }
        std::vector<int32_t> gsrc((size_t)gptr[(size_t)NR]);
        std::vector<uint32_t> gflag((size_t)gptr[(size_t)NR], 0u);
        {
            std::vector<int32_t> fill(gptr.begin(), gptr.end() - 1);
            for (int32_t l = 1; l <= B0; ++l) {
                const LayerPlan& lay = plan.layers[(size_t)l];
                for (int64_t p = 0; p < lay.n; ++p) {
                    const bool weighted = (l & 1) == 0 && lay.row_ptr[(size_t)p + 1] - lay.row_ptr[(size_t)p] > 1;
                    for (int32_t j = lay.row_ptr[(size_t)p]; j < lay.row_ptr[(size_t)p + 1]; ++j) {
                        const int32_t slot = fill[(size_t)lay.child[(size_t)j]]++;
                        gsrc[(size_t)slot] = (int32_t)(plan.row0[(size_t)l] + p);
                        if (weighted) gflag[(size_t)slot] = kWeightedEdge;
                    }
                }
            }
        }
        for (int32_t l = 0; l < B0; ++l) {
            // rows of layer l: a CSR slice rebased to start at 0
            const int64_t a = plan.row0[(size_t)l], n = plan.layers[(size_t)l].n;
            std::vector<int32_t> lptr((size_t)n + 1);
            for (int64_t i = 0; i <= n; ++i) lptr[(size_t)i] = gptr[(size_t)(a + i)] - gptr[(size_t)a];
            PassPlan& dst = plan.layers[(size_t)l + 1].bwd;
            // rows that are OR nodes with more than one child are flagged, as in the layer-by-layer plans
            make_pass_plan(n, lptr.data(), gsrc.data() + gptr[(size_t)a], popt, dst, gflag.data() + gptr[(size_t)a],
                           (l & 1) == 0 && l >= 2 ? plan.layers[(size_t)l].multi.data() : nullptr);
            plan.num_split_rows += dst.n_heavy;
            plan.max_bwd_seg = std::max<int64_t>(plan.max_bwd_seg, dst.n_seg);
        }
    }
    for (int32_t l = 0; l <= L; ++l) {
        plan.num_nodes += plan.layers[(size_t)l].n;
        plan.max_layer_nodes = std::max(plan.max_layer_nodes, plan.layers[(size_t)l].n);
    }

    // the narrow top: the longest suffix of layers that all kept their plain index vectors
    plan.tail_first = plan.tail_bwd_first = 0;
    if (!opt.no_tail) {
        int32_t t = L + 1;
        while (t - 1 >= 1 && plan.layers[(size_t)t - 1].tail_fwd_ok) --t;
        if (t <= L) plan.tail_first = t;
        t = L + 1;
        while (t - 1 >= 1 && plan.layers[(size_t)t - 1].tail_bwd_ok) --t;
        if (t <= L) plan.tail_bwd_first = t;
    }

    // ---------------------------------------------------------------- leaf layer and roots
    plan.num_vars = V;
    plan.num_roots = R;
    plan.num_layers = L;
    plan.pos_row.assign((size_t)V, -1);
    plan.neg_row.assign((size_t)V, -1);
    plan.leaf_code.resize((size_t)plan.layers[0].n);
    for (int64_t p = 0; p < plan.layers[0].n; ++p) {
        int32_t c = plan.layers[0].origin[(size_t)p];
        if (node_type[c] == T_LIT) {
            int32_t lit = node_lit[c];
            plan.leaf_code[(size_t)p] = lit;
            (lit > 0 ? plan.pos_row : plan.neg_row)[(size_t)(std::abs(lit) - 1)] = (int32_t)p;
        } else {
            plan.leaf_code[(size_t)p] = node_type[c] == T_TRUE ? INT32_MAX : INT32_MIN;
        }
    }
    plan.root_pos.resize((size_t)R);
    for (int32_t r = 0; r < R; ++r) plan.root_pos[(size_t)r] = at(roots[r], L);
    {
        const int64_t nt = plan.layers[(size_t)L].n;
        plan.top_ptr.assign((size_t)nt + 1, 0);
        plan.top_root.resize((size_t)R);
        for (int32_t r = 0; r < R; ++r) ++plan.top_ptr[(size_t)plan.root_pos[(size_t)r] + 1];
        for (int64_t i = 0; i < nt; ++i) plan.top_ptr[(size_t)i + 1] += plan.top_ptr[(size_t)i];
        std::vector<int32_t> fill(plan.top_ptr.begin(), plan.top_ptr.end() - 1);
        for (int32_t r = 0; r < R; ++r) plan.top_root[(size_t)fill[(size_t)plan.root_pos[(size_t)r]]++] = r;
    }
    return ST_OK;
}

}  // namespace klay
