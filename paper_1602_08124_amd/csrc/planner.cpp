// Step planner: policy -> ordered ops (Section 3.2) -> transfer windows -> lifetimes -> placement of the blocks
// in the pool; vDNN_dyn (Section 3.3) and the fit policy on top of it.  Pure host code.
#include "manager.h"

#include <algorithm>
#include <cstring>

#include "ops.h"

namespace vdnn {

// ---------------------------------------------------------------------------------------------
// planning
// ---------------------------------------------------------------------------------------------
namespace {

struct Compiler {
    const vdnn_net& n;
    Plan& p;
    size_t budget;  // aligned; SIZE_MAX/4 when unlimited
    size_t live = 0;
    int phase = 0, layer = -1;
    std::vector<size_t> samples;
    bool failed = false;

    Compiler(const vdnn_net& net, Plan& plan, size_t b) : n(net), p(plan), budget(b) {}

    std::string where() const {
        if (phase == 0) return "create";
        return fmt("%c%d", phase == 1 ? 'F' : 'B', layer);
    }

    Op& emit(OpKind k) {
        Op o;
        o.kind = k; o.phase = phase; o.layer = layer;
        p.ops.push_back(o);
        return p.ops.back();
    }

    int alloc(const std::string& tag, size_t raw, bool persistent = false) {
        Block b;
        b.tag = tag; b.raw = raw; b.bytes = align_up(std::max<size_t>(raw, 1));
        b.persistent = persistent;
        b.t0 = (int)p.ops.size(); b.t1 = -1;
        if (live + b.bytes > budget) {
            failed = true;
            p.fail_where = where();
            p.fail_why = fmt("%s: allocating %zu bytes for %s with %zu live exceeds the budget of %zu", where().c_str(), b.bytes,
                             tag.c_str(), live, budget);
            return -1;
        }
        live += b.bytes;
        p.peak = std::max(p.peak, live);
        p.blocks.push_back(b);
        const int id = (int)p.blocks.size() - 1;
        emit(OP_ALLOC).block = id;
        return id;
    }

    void release(int id) {
        live -= p.blocks[id].bytes;
        emit(OP_FREE).block = id;
        p.blocks[id].t1 = (int)p.ops.size();
    }
};

}  // namespace

// Placement of the transient blocks above the persistent region.  Blocks are taken in a priority
// order and each takes the lowest offset at which it overlaps no already placed block whose lifetime
// intersects its own.  The live-byte peak is the lower bound of the address range.  Four orders are
// tried first (by size; by lifetime; by size x lifetime; by allocation time); if none reaches the bound, the
// same priorities are perturbed with seeded noise for a bounded number of rounds and the best placement
// wins.  On the paper's workloads this reaches the bound (no fragmentation) within a few rounds.
//
// A block that moves in pieces occupies a staircase in (time x address): one rectangle per piece, at fixed
// distances from the block's offset.  It takes the lowest offset at which none of its rectangles meets a
// placed one; later blocks see its rectangles one by one and can move into the part of the range a piece
// has left (or not yet taken).
//
// A host, its tenants and its twin (see retime) form one such object too: the tenants' rectangles and the
// twin's staircase lie inside the host's range by construction, so the group is placed as a whole.
namespace {
struct Rect { size_t off, bytes; int t0, t1; };
struct Unit {
    std::vector<Rect> rects;                         // offsets relative to the unit's offset
    std::vector<std::pair<int, size_t>> members;     // (block, distance from the unit's offset)
    size_t bytes = 0;                                // address range the unit spans
    int t0 = 1 << 30, t1 = 0;
};
}

static std::vector<Unit> make_units(const Plan& p) {
    std::vector<Unit> units;
    std::vector<int> unit_of(p.blocks.size(), -1);
    auto add = [&](Unit& u, int id, size_t rel) {
        const Block& b = p.blocks[id];
        u.members.push_back({id, rel});
        for (int i = 0; i < b.parts; ++i) {
            const Rect r{rel + (b.parts == 1 ? 0 : (size_t)i * b.part_bytes), b.piece_bytes(i), b.parts == 1 ? b.t0 : b.part_t0[i],
                         b.parts == 1 ? b.t1 : b.part_t1[i]};
            u.rects.push_back(r);
            u.bytes = std::max(u.bytes, r.off + r.bytes);
            u.t0 = std::min(u.t0, r.t0);
            u.t1 = std::max(u.t1, r.t1);
        }
    };
    for (int id = 0; id < (int)p.blocks.size(); ++id) {
        if (p.blocks[id].persistent || p.blocks[id].host >= 0) continue;
        unit_of[id] = (int)units.size();
        units.emplace_back();
        add(units.back(), id, 0);
    }
    for (int id = 0; id < (int)p.blocks.size(); ++id)
        if (!p.blocks[id].persistent && p.blocks[id].host >= 0) add(units[unit_of[p.blocks[id].host]], id, p.blocks[id].host_rel);
    return units;
}

// limit: an order whose placement passes this extent is given up at once ((size_t)-1 is returned)
static size_t place_with_keys(const std::vector<Unit>& units, size_t n_blocks, size_t base, const std::vector<double>& key,
                              std::vector<size_t>& offsets, size_t limit = (size_t)-1) {
    std::vector<int> order(units.size());
    for (size_t i = 0; i < units.size(); ++i) order[i] = (int)i;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return key[a] > key[b]; });
    std::vector<Rect> placed;  // absolute offsets
    offsets.assign(n_blocks, 0);
    size_t extent = base;
    std::vector<std::pair<size_t, size_t>> conf;
    std::vector<Rect> near;
    for (int ui : order) {
        const Unit& u = units[ui];
        size_t off = base;
        if (u.rects.size() == 1) {
            conf.clear();
            for (const Rect& q : placed)
                if (q.t0 < u.t1 && u.t0 < q.t1) conf.push_back({q.off, q.bytes});
            std::sort(conf.begin(), conf.end());
            for (auto& c : conf) {
                if (off + u.bytes <= c.first) break;
                off = std::max(off, c.first + c.second);
            }
        } else {
            near.clear();
            for (const Rect& q : placed)
                if (q.t0 < u.t1 && u.t0 < q.t1) near.push_back(q);
            auto fits = [&](size_t o) {
                for (const Rect& r : u.rects)
                    for (const Rect& q : near)
                        if (q.t0 < r.t1 && r.t0 < q.t1 && o + r.off < q.off + q.bytes && q.off < o + r.off + r.bytes) return false;
                return true;
            };
            std::vector<size_t> cands{base};
            for (const Rect& r : u.rects)
                for (const Rect& q : near)
                    if (q.t0 < r.t1 && r.t0 < q.t1 && q.off + q.bytes >= base + r.off) cands.push_back(q.off + q.bytes - r.off);
            std::sort(cands.begin(), cands.end());
            for (size_t o : cands)
                if (fits(o)) { off = o; break; }   // sliding down from above every neighbour stops at one of the candidates
        }
        if (off + u.bytes > limit) return (size_t)-1;
        for (const Rect& r : u.rects) placed.push_back({off + r.off, r.bytes, r.t0, r.t1});
        for (auto& m : u.members) offsets[m.first] = off + m.second;
        extent = std::max(extent, off + u.bytes);
    }
    return extent;
}

// good_enough: the search stops at the first placement whose extent is at most this (0: only at the lower bound);
// rounds: how many perturbed orders are tried after the four plain ones.
// variant > 0: another placement of the same blocks: the plain orders are skipped and the perturbed ones drawn from a seed of
// their own; meant to be called with good_enough = the budget (the first placement that fits is returned).
static size_t place_blocks(Plan& p, size_t base, size_t good_enough = 0, int rounds = 300, uint64_t variant = 0) {
    const std::vector<Unit> units = make_units(p);
    if (units.empty()) return base;
    const size_t n = units.size();
    // lower bound of the extent: the largest number of bytes whose lifetimes (as placement sees them) overlap
    size_t bound = base;
    {
        std::vector<std::pair<int, long long>> ev;
        for (const Unit& u : units)
            for (const Rect& r : u.rects) { ev.push_back({r.t0, (long long)r.bytes}); ev.push_back({r.t1, -(long long)r.bytes}); }
        std::sort(ev.begin(), ev.end());   // at equal times releases (negative) come first: lifetimes are half-open
        long long live = 0, top = 0;
        for (auto& e : ev) { live += e.second; top = std::max(top, live); }
        bound = base + (size_t)top;
    }
    const size_t target = std::max(bound, good_enough);
    const size_t limit = good_enough ? good_enough : (size_t)-1;   // with a goal, orders that miss it need not be finished
    std::vector<double> size(n), life(n), area(n), start(n), key(n);
    for (size_t i = 0; i < n; ++i) {
        // ties: earlier blocks first (the sort is stable)
        size[i] = (double)units[i].bytes;
        life[i] = (double)(units[i].t1 - units[i].t0);
        area[i] = size[i] * life[i];
        start[i] = (double)(p.ops.size() + 2 - units[i].t0);  // allocation order: what a run-time first-fit allocator would do
    }
    std::vector<size_t> best, cur;
    size_t best_extent = (size_t)-1;
    constexpr int kKinds = 4;
    const std::vector<double>* base_keys[kKinds] = {&size, &life, &area, &start};
    for (int kind = 0; kind < kKinds && best_extent > target && !variant; ++kind) {
        const size_t e = place_with_keys(units, p.blocks.size(), base, *base_keys[kind], cur, limit);
        if (e < best_extent) { best_extent = e; best = cur; }
    }
    uint64_t rng = 0x9E3779B97F4A7C15ull + variant * 0xD1B54A32D192ED03ull;  // fixed seeds: the plan is a pure function of (net, policy, budget)
    auto next = [&]() { rng = rng * 6364136223846793005ull + 1442695040888963407ull; return (double)(rng >> 11) / 9007199254740992.0; };
    const double noises[4] = {0.1, 0.3, 0.6, 1.0};
    for (int round = 0; round < rounds && best_extent > target; ++round) {
        const std::vector<double>& k0 = *base_keys[(int)(next() * kKinds) % kKinds];
        const double noise = noises[(int)(next() * 4) % 4];
        for (size_t i = 0; i < n; ++i) key[i] = k0[i] * (1.0 + noise * (next() - 0.5));
        const size_t e = place_with_keys(units, p.blocks.size(), base, key, cur, limit);
        if (e < best_extent) { best_extent = e; best = cur; }
    }
    if (best_extent == (size_t)-1) return best_extent;   // no order stayed within the limit: offsets untouched
    for (const Unit& u : units)
        for (auto& m : u.members) p.blocks[m.first].offset = best[m.first];
    return best_extent;
}

// Compiles one training step under a static policy (NONE / ALL / CONV) and a convolution algorithm
// mode: performance-optimal everywhere, memory-optimal everywhere, or greedy (performance-optimal
// unless that layer's workspace would overflow the budget: Section 3.3, phase 3 of vDNN_dyn).
static void finish_plan(const vdnn_net& n, Plan& p, int fill_pm, int fill_bwd_pm, int place_rounds);

// offload_set (indexed by buffer id + 1), when given, replaces the policy's choice of feature maps;
// place = false stops after the byte accounting (p.ok then only says that the live total fits).
void compile_plan(const vdnn_net& n, int policy, int algo, Plan& p, const std::vector<char>* offload_set, bool place, int fill_pm,
                  int fill_bwd_pm, int place_rounds) {
    p = Plan();
    p.policy = policy;
    p.algo = algo;
    p.memopt_fwd.assign(n.layers.size(), 0);
    p.memopt_bwd.assign(n.layers.size(), 0);
    p.opt_fwd.assign(n.layers.size(), -1);
    p.opt_bwd.assign(n.layers.size(), -1);
    const size_t budget = n.budget ? n.budget / kAlign * kAlign : (size_t)-1 / 4;
    Compiler c(n, p, budget);
    const int L = (int)n.layers.size();
    std::vector<int> res(L + 1, -1), grad(L + 1, -1);        // buffer id + 1 -> block
    std::vector<char> on_host(L + 1, 0);
    std::vector<std::vector<int>> offloaded_at(L);            // layer -> buffers it offloaded
    std::vector<int> host_block(L + 1, -1);                   // buffer -> block it was offloaded from (for host_off)
    std::vector<int> w_block(L, -1), dw_block(L, -1);
    size_t pinned = 0;
    std::vector<size_t> host_off(L + 1, 0);
    // Which of a layer's options runs (Section 3.3): the performance-optimal one (the first), the memory-optimal one
    // (the last: no workspace), or, greedy, the first whose workspace fits the budget at this point of the step.
    auto choose = [&](const std::vector<KernelOption>& opts) -> int {
        if (opts.empty()) return -1;
        if (algo == VDNN_ALGO_MEM) return (int)opts.size() - 1;
        if (algo == VDNN_ALGO_GREEDY)
            for (size_t k = 0; k < opts.size(); ++k)
                if (!opts[k].ws || c.live + align_up(opts[k].ws) <= budget) return (int)k;
        return 0;
    };

#define CHECK_FAIL() do { if (c.failed) return; } while (0)

    // ---- create: persistent blocks --------------------------------------------------------
    c.phase = 0;
    for (int i = 0; i < L; ++i) {
        if (!n.layers[i].wcount) continue;
        w_block[i] = c.alloc(fmt("W%d", i), n.layers[i].wcount * 4, true); CHECK_FAIL();
        dw_block[i] = c.alloc(fmt("dW%d", i), n.layers[i].wcount * 4, true); CHECK_FAIL();
    }
    p.labels_block = c.alloc("labels", (size_t)n.batch * 4, true); CHECK_FAIL();
    p.loss_block = c.alloc("loss", 4, true); CHECK_FAIL();
    p.persistent = c.live;
    {   // persistent blocks are packed from offset 0 in creation order: their place never depends on the policy
        size_t off = 0;
        for (Block& b : p.blocks) { b.offset = off; off += b.bytes; b.t0 = 0; b.t1 = 1 << 30; }
    }

    // ---- forward --------------------------------------------------------------------------
    c.phase = 1; c.layer = -1;
    p.first_fwd_op = (int)p.ops.size();
    res[0] = c.alloc("B-1", n.B(-1).count * 4); CHECK_FAIL();
    p.blocks[res[0]].buf = -1;
    {
        Op& o = c.emit(OP_LOAD_INPUT);
        o.out_block = res[0];
    }
    for (int i = 0; i < L; ++i) {
        const Layer& l = n.layers[i];
        c.layer = i;
        c.emit(OP_SAMPLE);
        c.samples.push_back(c.live);
        if (!in_place(l.type) && l.type != VDNN_SOFTMAX_CE) { res[i + 1] = c.alloc(fmt("B%d", i), n.B(i).count * 4); CHECK_FAIL(); p.blocks[res[i + 1]].buf = i; }
        const int pick = choose(n.options_fwd[i]);
        const size_t ws = pick >= 0 ? n.options_fwd[i][pick].ws : 0;
        if (l.type == VDNN_CONV) {
            p.opt_fwd[i] = pick;
            p.memopt_fwd[i] = algo == VDNN_ALGO_MEM || (pick > 0 && pick == (int)n.options_fwd[i].size() - 1);
        }
        int wsb = -1;
        if (ws) { wsb = c.alloc("WS", ws); CHECK_FAIL(); p.max_ws = std::max(p.max_ws, ws); }
        std::vector<int> in_bufs;
        for (int src : l.inputs) in_bufs.push_back(buf_of(n, src));
        if (!in_place(l.type)) {
            for (int b : in_bufs) {
                if (n.B(b).readers.back() == i && (offload_set ? (bool)(*offload_set)[b + 1] : selected(n, b, policy))) {
                    Op& o = c.emit(OP_OFFLOAD);
                    o.block = res[b + 1]; o.buf = b;
                    host_off[b + 1] = pinned;
                    p.blocks[res[b + 1]].host_off = pinned;
                    pinned += align_up(n.B(b).count * 4);
                    p.offloaded += n.B(b).count * 4;
                    p.n_offload++;
                    offloaded_at[i].push_back(b);
                }
            }
        }
        {
            Op& o = c.emit(OP_FWD);
            for (int b : in_bufs) o.in_blocks.push_back(res[b + 1]);
            o.out_block = res[l.buf + 1];
            o.ws_block = wsb;
            if (l.type == VDNN_CONV) o.kern[0] = n.options_fwd[i][pick].fwd;
        }
        if (wsb >= 0) c.release(wsb);
        for (int b : offloaded_at[i]) {
            Op& o = c.emit(OP_WAIT_COPY);
            o.block = res[b + 1]; o.buf = b;
            c.release(res[b + 1]);
            res[b + 1] = -1;
            on_host[b + 1] = 1;
        }
        if (!in_place(l.type))
            for (int b : in_bufs)
                if (res[b + 1] >= 0 && n.B(b).readers.back() == i && n.B(b).bwd_users.empty()) { c.release(res[b + 1]); res[b + 1] = -1; }
    }

    // ---- backward -------------------------------------------------------------------------
    c.phase = 2;
    p.first_bwd_op = (int)p.ops.size();
    auto fetch = [&](int b, OpKind kind) -> bool {
        res[b + 1] = c.alloc(fmt("B%d", b), n.B(b).count * 4);
        if (c.failed) return false;
        p.blocks[res[b + 1]].buf = b;
        p.blocks[res[b + 1]].host_off = host_off[b + 1];
        on_host[b + 1] = 0;
        Op& o = c.emit(kind);
        o.block = res[b + 1]; o.buf = b;
        p.prefetched += n.B(b).count * 4;
        return true;
    };
    for (int m = L - 1; m >= 0; --m) {
        const Layer& l = n.layers[m];
        c.layer = m;
        c.emit(OP_SAMPLE);
        c.samples.push_back(c.live);
        // findPrefetchLayer (Fig. code_prefetch): nearest preceding layer whose offloaded X is still on the host;
        // the search window ends at the first CONV layer that has nothing to prefetch.
        std::vector<int> issued;
        for (int j = m - 1; j >= 0; --j) {
            std::vector<int> pending;
            for (int b : offloaded_at[j]) if (on_host[b + 1]) pending.push_back(b);
            if (!pending.empty()) {
                for (int b : pending) { if (!fetch(b, OP_PREFETCH)) return; p.n_prefetch++; issued.push_back(b); }
                break;
            }
            if (n.layers[j].type == VDNN_CONV) break;
        }
        std::vector<int> in_bufs;
        for (int src : l.inputs) in_bufs.push_back(buf_of(n, src));
        std::vector<int> needed;
        if (in_place(l.type)) needed.push_back(l.buf);
        else if (needs_x_in_bwd(l.type)) needed = in_bufs;
        for (int b : needed)
            if (on_host[b + 1]) { if (!fetch(b, OP_ONDEMAND)) return; p.n_ondemand++; }
        std::vector<int> gout(in_bufs.size(), -1), gacc(in_bufs.size(), -1), temps;
        if (!in_place(l.type)) {
            for (size_t k = 0; k < in_bufs.size(); ++k) {
                const int b = in_bufs[k];
                if (b < 0) continue;
                if (grad[b + 1] < 0) { grad[b + 1] = c.alloc(fmt("dB%d", b), n.B(b).count * 4); CHECK_FAIL(); gout[k] = grad[b + 1]; }
                else { const int t = c.alloc(fmt("T%d", b), n.B(b).count * 4); CHECK_FAIL(); temps.push_back(t); gout[k] = t; gacc[k] = grad[b + 1]; }
            }
        }
        const int pick = choose(n.options_bwd[m]);
        const size_t ws = pick >= 0 ? n.options_bwd[m][pick].ws : 0;
        if (l.type == VDNN_CONV) {
            p.opt_bwd[m] = pick;
            p.memopt_bwd[m] = algo == VDNN_ALGO_MEM || (pick > 0 && pick == (int)n.options_bwd[m].size() - 1);
        }
        int wsb = -1;
        if (ws) { wsb = c.alloc("WS", ws); CHECK_FAIL(); p.max_ws = std::max(p.max_ws, ws); }
        {
            Op& o = c.emit(OP_BWD);
            for (int b : in_bufs) o.in_blocks.push_back(res[b + 1]);
            o.out_block = l.type == VDNN_SOFTMAX_CE ? -1 : res[l.buf + 1];
            o.gin_block = l.type == VDNN_SOFTMAX_CE ? -1 : grad[l.buf + 1];
            o.gout_blocks = gout; o.gacc_blocks = gacc; o.ws_block = wsb;
            if (l.type == VDNN_CONV) { o.kern[1] = n.options_bwd[m][pick].bd; o.kern[2] = n.options_bwd[m][pick].bf; }
        }
        if (wsb >= 0) c.release(wsb);
        for (int t : temps) c.release(t);
        for (int b : issued) {  // end-of-layer synchronisation with the prefetch issued for this layer
            Op& o = c.emit(OP_WAIT_COPY);
            o.block = res[b + 1]; o.buf = b;
        }
        if (!in_place(l.type) && l.type != VDNN_SOFTMAX_CE) { c.release(grad[m + 1]); grad[m + 1] = -1; }
        for (int b = -1; b < L; ++b)
            if (res[b + 1] >= 0 && !n.B(b).bwd_users.empty() && n.B(b).bwd_users.front() == m) { c.release(res[b + 1]); res[b + 1] = -1; }
    }
#undef CHECK_FAIL
    p.pinned = pinned;
    p.w_block = w_block;
    p.dw_block = dw_block;
    p.offload_set.assign(L + 1, 0);
    for (int i = 0; i < L; ++i)
        for (int b : offloaded_at[i]) p.offload_set[b + 1] = 1;
    for (int i = 0; i < L; ++i)
        if (n.layers[i].type == VDNN_CONV && (p.memopt_fwd[i] || p.memopt_bwd[i])) p.n_memopt++;
    for (int i = 0; i < L; ++i) {
        if (n.layers[i].type != VDNN_CONV) continue;
        const KernelOption &f = n.options_fwd[i][p.opt_fwd[i]], &b = n.options_bwd[i][p.opt_bwd[i]];
        p.n_winograd += is_winograd(f.fwd) || is_winograd(b.bd) || is_winograd(b.bf);
        p.n_downgraded += algo == VDNN_ALGO_GREEDY && (p.opt_fwd[i] > 0 || p.opt_bwd[i] > 0);
    }
    if (place) finish_plan(n, p, fill_pm, fill_bwd_pm, place_rounds);
    else p.ok = true;
}

// Budget-aware transfer windows (not in the paper, which synchronises the two streams at the end of every
// layer: Section 3.2).  The transfers of the static schedule stay; what moves is when the pool gives up or
// takes the memory.
//   forward:  the release of an offloaded X (and the wait for its copy) is held back; held blocks queue in
//             copy order; an allocation that would pass `soft` first lets the oldest go, until the live total
//             fits.  The range of X is lent out while X is away: a feature map that is not offloaded itself
//             and had to let something go becomes a tenant of the block released last, lined up from the low
//             end of its range (pieces go from the low end upwards), and keeps letting pieces go until that
//             host has room for it; when a host runs out of pieces the next held block takes over.  The rest
//             go at the end of forward propagation;
//   backward: a block that moves in pieces is fetched from its top piece down, the mirror image of forward;
//             a fetch returns to the range its buffer had in forward propagation (as the host's twin) when
//             every tenant has left by then; the wait for a fetch moves to just before the first computation
//             that reads it.  Once the blocks have addresses, hoist_fetches moves every fetch (allocation +
//             copy), in the order of the static schedule, to the earliest point, not before the previous
//             fetch, from which its own address range is free and live bytes plus its size stay within
//             `soft_bwd`, up to its original place.
static void retime(const vdnn_net& n, Plan& p, size_t soft, size_t soft_bwd) {
    const int L = (int)n.layers.size();
    constexpr int kMaxParts = 32;
    // Blocks larger than the part size move in at most kMaxParts pieces of equal (aligned) size.
    auto split = [&](int block) {
        Block& b = p.blocks[block];
        if (!n.part_bytes || b.bytes <= n.part_bytes) return 1;
        const size_t k = std::min<size_t>(kMaxParts, (b.bytes + n.part_bytes - 1) / n.part_bytes);
        b.part_bytes = align_up((b.bytes + k - 1) / k);
        b.parts = (int)((b.bytes + b.part_bytes - 1) / b.part_bytes);
        return b.parts;
    };
    std::vector<Op> out;
    out.reserve(p.ops.size() + 64);
    for (int t = 0; t < p.first_fwd_op; ++t) out.push_back(p.ops[t]);
    size_t live = p.persistent;
    struct Held { Op wait, free; size_t bytes; };
    std::vector<Held> held;
    size_t held_head = 0;
    std::vector<size_t> released(p.blocks.size(), 0), taken(p.blocks.size(), 0);  // per host: bytes given up / lent so far
    std::vector<int> fwd_block_of(L + 1, -1);  // buffer id + 1 -> the block that was offloaded
    int host = -1;                             // block released last
    auto let_go = [&](int layer) {
        Held& h = held[held_head++];
        h.wait.layer = h.free.layer = layer;
        out.push_back(h.wait);
        out.push_back(h.free);
        live -= h.bytes;
        host = h.free.block;
        released[host] += h.bytes;
    };
    for (int t = p.first_fwd_op; t < p.first_bwd_op; ++t) {
        const Op& o = p.ops[t];
        if (o.kind == OP_OFFLOAD) {
            fwd_block_of[o.buf + 1] = o.block;
            const int k = split(o.block);
            for (int i = 0; i < k; ++i) {
                Op c = o;
                c.part = k == 1 ? -1 : i;
                out.push_back(c);
            }
            continue;
        }
        if (o.kind == OP_WAIT_COPY && t + 1 < p.first_bwd_op && p.ops[t + 1].kind == OP_FREE && p.ops[t + 1].block == o.block) {
            const Block& b = p.blocks[o.block];
            for (int i = 0; i < b.parts; ++i) {
                Held h{o, p.ops[t + 1], b.piece_bytes(i)};
                h.wait.part = h.free.part = b.parts == 1 ? -1 : i;
                held.push_back(h);
            }
            ++t;
            continue;
        }
        if (o.kind == OP_ALLOC) {
            const size_t s = p.blocks[o.block].bytes;
            if (live + s > soft) {
                // a feature map that is not offloaded itself moves into the range of the block released last
                Block& me = p.blocks[o.block];
                const bool rents = me.buf >= -1 && !p.offload_set[me.buf + 1];
                auto room = [&]() { return host >= 0 ? released[host] - taken[host] : (size_t)0; };
                while (held_head < held.size() && (live + s > soft || (rents && room() < s))) let_go(o.layer);
                if (rents && room() >= s) {
                    me.host = host;
                    me.host_rel = taken[host];
                    taken[host] += s;
                }
            }
            live += s;
        } else if (o.kind == OP_FREE) {
            live -= p.blocks[o.block].bytes;
        }
        out.push_back(o);
    }
    // With backward windows the copies still queued at the end of forward propagation stay queued: their blocks are
    // released in backward propagation, oldest first, when an allocation there needs the room (at the latest before the
    // same feature map is fetched again).  Forward propagation then ends with its last computation, not with its last
    // copy.  Without backward windows everything queued is released here.
    const bool trailing = soft_bwd > 0;
    if (!trailing)
        while (held_head < held.size()) let_go(L - 1);
    const int new_first_bwd = (int)out.size();

    // backward: fetches stay where the static schedule has them (hoist_fetches moves them once the blocks have
    // addresses), but are cut into pieces, top piece first, and awaited just before their first reader
    const std::vector<Op> bw(p.ops.begin() + p.first_bwd_op, p.ops.end());
    const int nb = (int)bw.size();
    std::vector<int> freed_at(p.blocks.size(), -1);  // block -> backward op that releases it
    for (int t = 0; t < nb; ++t)
        if (bw[t].kind == OP_FREE) freed_at[bw[t].block] = t;
    std::vector<std::vector<int>> await(p.blocks.size());  // block -> pieces whose copy the first reader has to wait for
    std::vector<char> waited(p.blocks.size(), 0);
    auto let_go_bwd = [&](int layer) {
        Held& h = held[held_head++];
        h.wait.layer = h.free.layer = layer;
        h.wait.phase = h.free.phase = 2;
        out.push_back(h.wait);
        out.push_back(h.free);
        live -= h.bytes;
    };
    auto make_room = [&](size_t s, int layer) {
        while (held_head < held.size() && live + s > soft_bwd) let_go_bwd(layer);
    };
    for (int t = 0; t < nb; ++t) {
        const Op& o = bw[t];
        if (o.kind == OP_ALLOC && t + 1 < nb && (bw[t + 1].kind == OP_PREFETCH || bw[t + 1].kind == OP_ONDEMAND) && bw[t + 1].block == o.block) {
            const int block = o.block;
            const int k = split(block);
            const int fwd_block = fwd_block_of[p.blocks[block].buf + 1];
            // a feature map comes back only after the copy of it that forward propagation made has left the pool
            if (fwd_block >= 0) {
                size_t last = held_head;
                for (size_t i = held_head; i < held.size(); ++i)
                    if (held[i].free.block == fwd_block) last = i + 1;
                while (held_head < last) let_go_bwd(o.layer);
            }
            // the fetch returns to the range its buffer had in forward propagation when every tenant has left by then
            if (fwd_block >= 0) {
                bool any = false, gone = true;
                for (size_t b = 0; b < p.blocks.size(); ++b)
                    if (p.blocks[b].host == fwd_block) { any = true; gone = gone && freed_at[b] < t; }  // -1: released in forward already
                if (any && gone) { p.blocks[block].host = fwd_block; p.blocks[block].host_rel = 0; }
            }
            for (int i = k - 1; i >= 0; --i) {
                Op a = o, c = bw[t + 1];
                a.part = c.part = k == 1 ? -1 : i;
                const size_t s = p.blocks[block].piece_bytes(i);
                make_room(s, o.layer);
                live += s;
                out.push_back(a);
                out.push_back(c);
                if (c.kind == OP_PREFETCH) await[block].push_back(c.part);  // an on-demand fetch waits by itself
            }
            ++t;
            continue;
        }
        if (o.kind == OP_WAIT_COPY && !await[o.block].empty()) continue;  // re-issued below, before the first reader
        if (o.kind == OP_BWD) {
            std::vector<int> reads = o.in_blocks;
            reads.push_back(o.out_block);
            for (int b : reads)
                if (b >= 0 && !await[b].empty() && !waited[b]) {
                    for (int part : await[b]) {
                        Op w;
                        w.kind = OP_WAIT_COPY; w.phase = 2; w.layer = o.layer; w.block = b; w.part = part;
                        out.push_back(w);
                    }
                    waited[b] = 1;
                }
        }
        if (o.kind == OP_ALLOC) {
            make_room(p.blocks[o.block].bytes, o.layer);
            live += p.blocks[o.block].bytes;
        } else if (o.kind == OP_FREE) {
            live -= p.blocks[o.block].bytes;
        }
        out.push_back(o);
    }
    while (held_head < held.size()) let_go_bwd(0);   // nothing is left here when every offloaded feature map is fetched again
    p.ops.swap(out);
    p.first_bwd_op = new_first_bwd;
}

// Lifetimes of blocks and pieces in op indices, live-byte statistics and copy counts of the op list.
static void measure_plan(Plan& p) {
    size_t live = 0;
    double sum = 0.0;
    size_t n_samples = 0;
    p.peak = 0; p.n_offload = p.n_prefetch = p.n_ondemand = 0;
    for (Block& b : p.blocks) {
        b.t0 = b.t1 = -1;
        b.part_t0.assign(b.parts, -1);
        b.part_t1.assign(b.parts, -1);
    }
    for (int t = 0; t < (int)p.ops.size(); ++t) {
        const Op& o = p.ops[t];
        if (o.kind == OP_ALLOC || o.kind == OP_FREE) {
            Block& b = p.blocks[o.block];
            const size_t bytes = o.part < 0 ? b.bytes : b.piece_bytes(o.part);
            for (int i = 0; i < b.parts; ++i) {
                if (o.part >= 0 && i != o.part) continue;
                if (o.kind == OP_ALLOC) b.part_t0[i] = t; else b.part_t1[i] = t + 1;
            }
            if (o.kind == OP_ALLOC) { if (b.t0 < 0) b.t0 = t; live += bytes; p.peak = std::max(p.peak, live); }
            else { b.t1 = t + 1; live -= bytes; }
        }
        else if (o.kind == OP_SAMPLE) { sum += (double)live; ++n_samples; }
        else if (o.kind == OP_OFFLOAD) p.n_offload++;   // copies issued: a block that moves in pieces counts once per piece
        else if (o.kind == OP_PREFETCH) p.n_prefetch++;
        else if (o.kind == OP_ONDEMAND) p.n_ondemand++;
    }
    const int t_end = (int)p.ops.size() + 1;
    for (Block& b : p.blocks) {
        if (b.persistent) { b.t0 = 0; b.t1 = 1 << 30; }
        else if (b.t1 < 0) b.t1 = t_end;  // still live at the end of the step (nothing should be)
        for (int i = 0; i < b.parts; ++i) {
            if (b.persistent) { b.part_t0[i] = 0; b.part_t1[i] = 1 << 30; }
            else if (b.part_t1[i] < 0) b.part_t1[i] = t_end;
        }
    }
    p.avg = n_samples ? sum / (double)n_samples : 0.0;
}

namespace {
struct Span { size_t off, bytes; int t0, t1, block; };
}
static std::vector<Span> spans_of(const Plan& p) {
    std::vector<Span> v;
    for (int id = 0; id < (int)p.blocks.size(); ++id) {
        const Block& b = p.blocks[id];
        if (b.persistent) continue;
        for (int i = 0; i < b.parts; ++i)
            v.push_back({b.offset + (b.parts == 1 ? 0 : (size_t)i * b.part_bytes), b.piece_bytes(i), b.parts == 1 ? b.t0 : b.part_t0[i],
                         b.parts == 1 ? b.t1 : b.part_t1[i], id});
    }
    return v;
}

// True when two pieces of memory that are live at the same time share an address.
static bool plan_overlaps(const Plan& p) {
    const std::vector<Span> v = spans_of(p);
    for (size_t i = 0; i < v.size(); ++i)
        for (size_t j = i + 1; j < v.size(); ++j)
            if (v[i].t0 < v[j].t1 && v[j].t0 < v[i].t1 && v[i].off < v[j].off + v[j].bytes && v[j].off < v[i].off + v[i].bytes) return true;
    return false;
}

// Early fetches, after placement (see retime).  A fetch (or a piece of one) sits at address range R from op q
// of the static schedule.  It may start at any earlier op from which R is free: nothing else that the
// placement put into R is live then.  Because every other block keeps its address and its lifetime, the
// placement stays valid, and the pool's extent does not change.
static void hoist_fetches(Plan& p, size_t soft_bwd) {
    const std::vector<Span> spans = spans_of(p);
    const int f0 = p.first_bwd_op, nt = (int)p.ops.size();
    std::vector<size_t> before(nt + 1, 0);  // live bytes before each op
    {
        size_t live = 0;
        for (int t = 0; t < nt; ++t) {
            before[t] = live;
            const Op& o = p.ops[t];
            if (o.kind != OP_ALLOC && o.kind != OP_FREE) continue;
            const Block& b = p.blocks[o.block];
            const size_t bytes = o.part < 0 ? b.bytes : b.piece_bytes(o.part);
            if (o.kind == OP_ALLOC) live += bytes; else live -= bytes;
        }
    }
    std::vector<std::vector<int>> landing(nt + 1);
    std::vector<char> skip(nt + 1, 0);
    int lo = f0;
    for (int q = f0; q + 1 < nt; ++q) {
        const Op& a = p.ops[q];
        const Op& c = p.ops[q + 1];
        if (a.kind != OP_ALLOC || (c.kind != OP_PREFETCH && c.kind != OP_ONDEMAND) || c.block != a.block || c.part != a.part) continue;
        const Block& b = p.blocks[a.block];
        const size_t s = a.part < 0 ? b.bytes : b.piece_bytes(a.part);
        const size_t r0 = b.offset + (a.part < 0 ? 0 : (size_t)a.part * b.part_bytes), r1 = r0 + s;
        int ready = lo;
        for (const Span& v : spans) {
            if (v.block == a.block || v.t0 >= q) continue;
            // not before whatever lies in its range has gone, nor before the copy of the same feature map that forward
            // propagation made has been released (its offload is what the fetch reads back)
            if ((v.off < r1 && r0 < v.off + v.bytes) || p.blocks[v.block].buf == b.buf) ready = std::max(ready, v.t1);
        }
        int j = q;
        while (j > ready && before[j - 1] + s <= soft_bwd) --j;
        if (j < q) {
            for (int t = j; t <= q; ++t) before[t] += s;
            landing[j].push_back(q);
            skip[q] = skip[q + 1] = 1;
            lo = j;
        } else {
            lo = q + 2;
        }
    }
    std::vector<Op> out;
    out.reserve(p.ops.size() + 32);
    auto emit_landing = [&](int t) {
        for (int q : landing[t]) {
            Op a = p.ops[q], c = p.ops[q + 1];
            a.layer = c.layer = p.ops[t].layer;
            c.kind = OP_PREFETCH;
            out.push_back(a);
            out.push_back(c);
        }
    };
    for (int t = 0; t < nt; ++t) {
        const Op& o = p.ops[t];
        if (o.kind != OP_SAMPLE) emit_landing(t);
        if (!skip[t]) out.push_back(o);
        else if (o.kind == OP_ONDEMAND) {  // the copy left: what stays is the wait that an on-demand fetch implies
            Op w = o;
            w.kind = OP_WAIT_COPY;
            out.push_back(w);
        }
        if (o.kind == OP_SAMPLE) emit_landing(t);
    }
    p.ops.swap(out);
}

// Before placement: how early could each fetch start if only live bytes counted?  The answer is written into the
// lifetimes that placement sees (not into the op list), so that placement keeps the fetch's address range clear
// from then on and hoist_fetches finds it free.  Inside a host's range the tenants still come first: a piece of a
// twin cannot start before the tenants that overlap it have left.  Returns whether any lifetime was extended.
static bool reserve_fetch_ranges(Plan& p, size_t soft_bwd) {
    const int f0 = p.first_bwd_op, nt = (int)p.ops.size();
    std::vector<size_t> before(nt + 1, 0);
    {
        size_t live = 0;
        for (int t = 0; t < nt; ++t) {
            before[t] = live;
            const Op& o = p.ops[t];
            if (o.kind != OP_ALLOC && o.kind != OP_FREE) continue;
            const Block& b = p.blocks[o.block];
            const size_t bytes = o.part < 0 ? b.bytes : b.piece_bytes(o.part);
            if (o.kind == OP_ALLOC) live += bytes; else live -= bytes;
        }
    }
    bool any = false;
    int lo = f0;
    for (int q = f0; q + 1 < nt; ++q) {
        const Op& a = p.ops[q];
        const Op& c = p.ops[q + 1];
        if (a.kind != OP_ALLOC || (c.kind != OP_PREFETCH && c.kind != OP_ONDEMAND) || c.block != a.block || c.part != a.part) continue;
        Block& b = p.blocks[a.block];
        const size_t s = a.part < 0 ? b.bytes : b.piece_bytes(a.part);
        int ready = lo;
        for (int id = 0; id < (int)p.blocks.size(); ++id) {   // after the forward copy of the same feature map has been released
            const Block& t = p.blocks[id];
            if (id != a.block && !t.persistent && t.buf == b.buf && t.t0 < q) ready = std::max(ready, t.t1);
        }
        if (b.host >= 0) {
            const size_t r0 = b.host_rel + (a.part < 0 ? 0 : (size_t)a.part * b.part_bytes), r1 = r0 + s;
            for (int id = 0; id < (int)p.blocks.size(); ++id) {
                const Block& t = p.blocks[id];
                if (id == a.block || t.host != b.host || t.t0 >= q) continue;
                if (t.host_rel < r1 && r0 < t.host_rel + t.bytes) ready = std::max(ready, t.t1);
            }
        }
        int j = q;
        while (j > ready && before[j - 1] + s <= soft_bwd) --j;
        if (j < q) {
            for (int t = j; t <= q; ++t) before[t] += s;
            if (a.part < 0) b.t0 = j;
            else { b.part_t0[a.part] = j; b.t0 = std::min(b.t0, j); }
            any = true;
            lo = j;
        } else {
            lo = q + 2;
        }
    }
    return any;
}

// Second half of planning: optional transfer windows, then lifetimes, statistics and placement.
static void finish_plan(const vdnn_net& n, Plan& p, int fill_pm, int fill_bwd_pm, int place_rounds) {
    const size_t budget = n.budget ? n.budget / kAlign * kAlign : (size_t)-1 / 4;
    p.ok = false;
    p.fill_pm = p.fill_bwd_pm = 0;
    // budget * fill / 1000 rounded down to a block boundary, in integers
    auto soft = [&](int pm) { return (size_t)((unsigned __int128)budget * (unsigned)pm / 1000u) / kAlign * kAlign; };
    const bool windows = (fill_pm > 0 || fill_bwd_pm > 0) && n.budget;
    if (windows) {
        retime(n, p, soft(fill_pm), fill_bwd_pm > 0 ? soft(fill_bwd_pm) : 0);
        p.fill_pm = fill_pm;
    }
    measure_plan(p);
    p.extent = place_blocks(p, p.persistent, 0, place_rounds);
    if (p.extent > budget) {
        p.fail_where = "placement";
        p.fail_why = fmt("live bytes peak at %zu but no placement of the blocks fits %zu (needs %zu)", p.peak, budget, p.extent);
        return;
    }
    if (windows && fill_bwd_pm > 0) {
        // How early a fetch can be issued depends on where the blocks lie (hoist_fetches).  A step that can be placed is
        // therefore placed again with the ranges of the fetches kept clear from as early as live bytes allow (for the whole
        // share of the budget, then for less).  Without a profile the first such placement that fits the budget replaces
        // the plain one.  With a profile every placement that fits is a candidate, together with further placements from
        // perturbed orders, and the one whose hoisted schedule has the shortest estimated step is taken.
        static const int kReserve[] = {1000, 900, 800};
        const int rounds = p.blocks.size() <= 600 ? place_rounds : 0;
        const bool by_time = n.profiled && place_rounds >= 100;
        auto offsets_of = [](const Plan& q) {
            std::vector<size_t> v(q.blocks.size());
            for (size_t i = 0; i < q.blocks.size(); ++i) v[i] = q.blocks[i].offset;
            return v;
        };
        std::vector<std::pair<std::vector<size_t>, size_t>> cands;   // (offsets, extent)
        cands.push_back({offsets_of(p), p.extent});
        for (int pm : kReserve) {
            if (pm > fill_bwd_pm) continue;
            Plan q = p;
            if (!reserve_fetch_ranges(q, soft(pm))) break;
            const int variants = by_time ? 6 : 0;
            bool fits = false;
            for (int v = 0; v <= variants; ++v) {
                Plan r = q;
                const size_t e = place_blocks(r, r.persistent, budget, rounds, (uint64_t)v);
                if (e <= budget) { cands.push_back({offsets_of(r), e}); fits = true; }
            }
            if (fits && !by_time) break;
        }
        if (by_time)
            for (int v = 1; v <= 6; ++v) {
                Plan r = p;
                const size_t e = place_blocks(r, r.persistent, budget, rounds, (uint64_t)v);
                if (e <= budget) cands.push_back({offsets_of(r), e});
            }
        const Plan kept = p;
        Plan best;
        double best_ms = -1.0;
        // without a profile: the last candidate is the reserved placement (when one fits), else the plain one
        for (size_t c = by_time ? 0 : cands.size() - 1; c < cands.size(); ++c) {
            Plan t = kept;
            for (size_t i = 0; i < t.blocks.size(); ++i) t.blocks[i].offset = cands[c].first[i];
            t.extent = cands[c].second;
            hoist_fetches(t, soft(fill_bwd_pm));
            measure_plan(t);
            if (plan_overlaps(t)) continue;  // cannot happen by construction; a plan that fails the check is never run
            t.fill_bwd_pm = fill_bwd_pm;
            t.ok = true;
            const double ms = by_time ? estimate_step_ms(n, t) : 0.0;
            if (best_ms < 0 || ms < best_ms) { best = t; best_ms = ms; }
        }
        if (best_ms >= 0) p = best;
    }
    p.ok = true;
}

// Estimated duration of a planned step from the profile (Section 3.3: vDNN_dyn decides from measured layer times; Section 3.2,
// Fig. vdnn_fwd / vdnn_bwd: the step is a compute timeline and a memory timeline -- here one per direction of the link --
// tied together where a transfer starts and where the computation waits for it).  Replays the op list: a computation takes
// its layer's measured time; a copy starts when its stream is free and everything enqueued before it on the compute stream
// has finished, and takes bytes / link rate; a wait moves the compute stream to the end of that copy.  < 0: no profile.
double estimate_step_ms(const vdnn_net& n, const Plan& p) {
    if (!n.profiled || !p.ok) return -1.0;
    const double d2h = (n.link_d2h_gbps > 0 ? n.link_d2h_gbps : 55.0) * 1e6, h2d = (n.link_h2d_gbps > 0 ? n.link_h2d_gbps : 55.0) * 1e6;  // bytes per ms
    // a kernel that was not measured is taken to be twice as slow as the slowest one of its pass that was
    auto conv_ms = [&](int i, int pass, int k) -> double {
        const LayerProfile& pr = n.profile[i];
        if (pr.conv[pass][k] >= 0) return pr.conv[pass][k];
        double worst = 0.0;
        for (int j = 0; j < kNumKernels; ++j) worst = std::max(worst, (double)pr.conv[pass][j]);
        return 2.0 * worst;
    };
    // the kernels come from the plan's own ops (the lists they were chosen from are re-sorted whenever the profile changes)
    auto fwd_ms = [&](const Op& o) -> double {
        const int i = o.layer;
        if (n.layers[i].type != VDNN_CONV) return n.profile[i].fwd > 0 ? n.profile[i].fwd : 0.0;
        return conv_ms(i, kPassFwd, o.kern[0]);
    };
    auto bwd_ms = [&](const Op& o) -> double {
        const int i = o.layer;
        if (n.layers[i].type != VDNN_CONV) return n.profile[i].bwd > 0 ? n.profile[i].bwd : 0.0;
        return conv_ms(i, kPassBwdFilter, o.kern[2]) + (buf_of(n, n.layers[i].inputs[0]) >= 0 ? conv_ms(i, kPassBwdData, o.kern[1]) : 0.0);
    };
    constexpr int kSlots = 33;
    std::vector<double> copy_end(p.blocks.size() * kSlots, 0.0);
    double tc = 0.0, tm_out = 0.0, tm_in = 0.0;   // compute stream; offloads and fetches each have a stream (and a link direction) of their own
    for (int t = p.first_fwd_op; t < (int)p.ops.size(); ++t) {
        const Op& o = p.ops[t];
        switch (o.kind) {
            case OP_FWD: tc += fwd_ms(o); break;
            case OP_BWD: tc += bwd_ms(o); break;
            case OP_OFFLOAD:
            case OP_PREFETCH:
            case OP_ONDEMAND: {
                const Block& b = p.blocks[o.block];
                const double bytes = (double)(o.part < 0 ? b.raw : b.piece_raw(o.part));
                double& tm = o.kind == OP_OFFLOAD ? tm_out : tm_in;
                const double end = std::max(tm, tc) + bytes / (o.kind == OP_OFFLOAD ? d2h : h2d);
                tm = end;
                copy_end[(size_t)o.block * kSlots + o.part + 1] = end;
                if (o.kind == OP_ONDEMAND) tc = std::max(tc, end);
                break;
            }
            case OP_WAIT_COPY: tc = std::max(tc, copy_end[(size_t)o.block * kSlots + o.part + 1]); break;
            default: break;
        }
    }
    return std::max(tc, std::max(tm_out, tm_in));
}

// Section 3.3, "Dynamic vDNN".  Trainability of a pass is decided by the planner, which performs
// exactly the allocations a real pass would (the paper's profiling passes only use pass/fail).
//   1. all with the memory-optimal algorithm: can the network be trained at all;
//   2. performance-optimal algorithms without offloading, else with conv, else with all;
//   3. greedy per-layer algorithm downgrade under conv, then under all; else back to 1.
//
// VDNN_POLICY_FIT is not one of the paper's policies.  It takes the observation behind vDNN_dyn (offload no
// more than the budget asks for) one step further: the offload set is built from single feature maps, and the
// transfers get budget-aware windows (see retime).
static bool fits_with(const vdnn_net& n, const std::vector<char>& set, int algo) {
    Plan q;
    compile_plan(n, VDNN_POLICY_FIT, algo, q, &set, false);
    return q.ok;
}

// Start with nothing offloaded.  While the step does not fit: add the smallest remaining candidate whose
// addition makes it fit; if there is none, add the largest remaining one (ties: lower id) and repeat.
static bool fit_select(const vdnn_net& n, int algo, std::vector<char>& set) {
    const int L = (int)n.layers.size();
    std::vector<int> cands;
    for (int b = -1; b < L; ++b)
        if (n.B(b).count && selected(n, b, VDNN_POLICY_ALL)) cands.push_back(b);
    set.assign(L + 1, 0);
    while (!fits_with(n, set, algo)) {
        std::vector<int> rest;
        for (int b : cands)
            if (!set[b + 1]) rest.push_back(b);
        if (rest.empty()) return false;
        std::stable_sort(rest.begin(), rest.end(), [&](int a, int b) { return n.B(a).count < n.B(b).count; });
        bool done = false;
        for (int b : rest) {
            set[b + 1] = 1;
            if (fits_with(n, set, algo)) { done = true; break; }
            set[b + 1] = 0;
        }
        if (done) break;
        int pick = rest[0];
        for (int b : rest)
            if (n.B(b).count > n.B(pick).count) pick = b;  // rest is ascending by (size, id): the first of the largest wins
        set[pick + 1] = 1;
    }
    return true;
}

// With a profile, the byte-driven choice above is only the starting point: which feature maps are away decides when the
// link is busy and when memory is short, and sets of equal size differ in how well their transfers hide behind the layers
// (Section 3.1: reuse distance).  Local search on the estimated step time: exchange one member for one non-member, or for two
// of about its size together, add one, or drop one; a move is taken when the step still fits and the estimate improves by half a per cent
// or more; until no move does (at most four rounds).  Candidates are what vDNN_all would offload.
static const int kSearchFills[] = {1000, 970, 950, 900, 800, 0};

// place_rounds: 12 for a candidate of the search (few placement rounds each); the default effort for a plan that must not be
// missed (the greedy mode fills the pool to the brim, and such a step needs more rounds to place)
static bool plan_with_windows(const vdnn_net& n, int algo, const std::vector<char>& set, Plan& out, int place_rounds = 12) {
    if (!fits_with(n, set, algo)) return false;
    for (int f : kSearchFills) {
        compile_plan(n, VDNN_POLICY_FIT, algo, out, &set, true, f, f ? 1000 : 0, place_rounds);
        if (out.ok) return true;
    }
    return false;
}

static void improve_by_time(const vdnn_net& n, int algo, std::vector<char>& set, Plan& best) {
    const int L = (int)n.layers.size();
    std::vector<int> cands;
    for (int b = -1; b < L; ++b)
        if (n.B(b).count && selected(n, b, VDNN_POLICY_ALL)) cands.push_back(b);
    double best_ms = estimate_step_ms(n, best);
    // Planning a candidate costs time in proportion to the step's blocks (VGG-16: 2 ms, VGG-116: 0.3 s), so the search gets a
    // budget of candidate plans that shrinks with the graph: the few hundred that VGG-16's neighbourhoods hold, a few dozen
    // for a net of hundreds of layers, where it is spent on the first moves in a fixed order (dropping a member, then exchanges).
    long long budget = std::max<long long>(24, std::min<long long>(400, 60000 / std::max<size_t>(1, best.blocks.size())));
    Plan q;
    for (int round = 0; round < 4 && budget > 0; ++round) {
        std::vector<char> round_set = set;
        double round_ms = best_ms;
        Plan round_plan;
        auto consider = [&](const std::vector<char>& t) {
            if (budget <= 0) return;
            --budget;
            if (!plan_with_windows(n, algo, t, q)) return;
            const double ms = estimate_step_ms(n, q);
            if (ms < round_ms) { round_ms = ms; round_set = t; round_plan = q; }
        };
        std::vector<int> in, out;
        for (int b : cands) (set[b + 1] ? in : out).push_back(b);
        // members from the smallest up: exchanging a small member has few candidates, and the budget should not run out on
        // the many pairs that could stand in for the largest one before the small ones have had their turn
        std::stable_sort(in.begin(), in.end(), [&](int a, int b) { return n.B(a).count < n.B(b).count; });
        for (int m : in) {
            std::vector<char> t = set;
            t[m + 1] = 0;
            consider(t);                                    // drop one
        }
        for (int m : in) {
            std::vector<char> t = set;
            t[m + 1] = 0;
            for (size_t i = 0; i < out.size(); ++i) {
                t[out[i] + 1] = 1;
                consider(t);                                // one for one
                for (size_t j = i + 1; j < out.size(); ++j) {
                    const size_t both = n.B(out[i]).count + n.B(out[j]).count;
                    if (2 * both < n.B(m).count || 4 * both > 5 * n.B(m).count) continue;   // two for one: 50 .. 125 % of its size
                    t[out[j] + 1] = 1;
                    consider(t);
                    t[out[j] + 1] = 0;
                }
                t[out[i] + 1] = 0;
            }
        }
        for (int a : out) {
            std::vector<char> t = set;
            t[a + 1] = 1;
            consider(t);                                    // add one
        }
        if (round_ms > best_ms * 0.995) break;
        set = round_set; best = round_plan; best_ms = round_ms;
    }
}

static const int kFills[] = {1000, 990, 980, 970, 960, 950, 940, 930, 920, 910, 900, 880, 860, 840, 820, 800, 750, 700, 600, 500, 0};

vdnn_status_t plan_policy(vdnn_net& n, int policy) {
    Plan p;
    if (policy == VDNN_POLICY_FIT) {
        std::vector<char> set;
        int algo = -1;
        for (int a : {VDNN_ALGO_PERF, VDNN_ALGO_GREEDY, VDNN_ALGO_MEM})
            if (fit_select(n, a, set)) { algo = a; break; }
        if (algo < 0) { n.err = "fit: the step does not fit even with every CONV/POOL input offloaded and no workspace"; return VDNN_ERR_OOM_DEVICE; }
        // The set was chosen by live bytes; when no placement of the blocks fits the budget either (the live
        // peak then sits within a fraction of a percent of it), the largest remaining candidate is added.
        bool planned = false;
        while (!planned) {
            // the largest forward share for which the blocks can be placed (the backward windows come out of the
            // placement and never make it fail)
            for (int f : kFills) {
                compile_plan(n, policy, algo, p, &set, true, f, f ? 1000 : 0);
                if (p.ok) { planned = true; break; }
            }
            if (planned) break;
            int pick = -2;
            for (int b = -1; b < (int)n.layers.size(); ++b)
                if (n.B(b).count && selected(n, b, VDNN_POLICY_ALL) && !set[b + 1] && (pick == -2 || n.B(b).count > n.B(pick).count)) pick = b;
            if (pick == -2) break;
            set[pick + 1] = 1;
        }
        if (!planned) { n.err = p.fail_why; return VDNN_ERR_OOM_DEVICE; }
        if (n.profiled && n.budget && p.blocks.size() <= 2000) {   // (the largest graphs keep the byte-driven set: planning time)
            improve_by_time(n, algo, set, p);
            // The greedy mode gives up a fast kernel where its workspace does not fit; that can let a smaller set of feature
            // maps do, and on a slow link the bytes saved outweigh the slower kernels.  Both are planned; the estimate decides.
            if (algo == VDNN_ALGO_PERF && p.blocks.size() <= 600) {   // (not for the largest graphs: planning time)
                std::vector<char> gset;
                Plan g;
                if (fit_select(n, VDNN_ALGO_GREEDY, gset) && plan_with_windows(n, VDNN_ALGO_GREEDY, gset, g, 300)) {
                    improve_by_time(n, VDNN_ALGO_GREEDY, gset, g);
                    if (estimate_step_ms(n, g) < 0.995 * estimate_step_ms(n, p)) { p = g; set = gset; algo = VDNN_ALGO_GREEDY; }
                }
            }
            // the winner once more with the full placement effort
            Plan fin;
            for (int f : kFills) {
                compile_plan(n, policy, algo, fin, &set, true, f, f ? 1000 : 0);
                if (fin.ok) break;
            }
            if (fin.ok && estimate_step_ms(n, fin) <= estimate_step_ms(n, p)) p = fin;
        }
        n.plan = p; n.policy = policy; n.effective = policy;
        return VDNN_OK;
    }
    if (policy == VDNN_POLICY_DYN) {
        Plan first;
        compile_plan(n, VDNN_POLICY_ALL, VDNN_ALGO_MEM, first);
        if (!first.ok) { n.err = "vDNN_dyn: even vDNN_all with the memory-optimal algorithm does not fit: " + first.fail_why; return VDNN_ERR_OOM_DEVICE; }
        if (n.profiled) {
            // With measured layer times and link rates the passes need not be tried in a fixed order that stands in for
            // "fastest first": every configuration of phases 2 and 3 (and no offloading with the greedy downgrade, which
            // the paper's order never reaches) is planned, and the one with the shortest estimated step is adopted.
            static const int cands[6][2] = {{VDNN_POLICY_NONE, VDNN_ALGO_PERF}, {VDNN_POLICY_CONV, VDNN_ALGO_PERF}, {VDNN_POLICY_ALL, VDNN_ALGO_PERF},
                                            {VDNN_POLICY_NONE, VDNN_ALGO_GREEDY}, {VDNN_POLICY_CONV, VDNN_ALGO_GREEDY}, {VDNN_POLICY_ALL, VDNN_ALGO_GREEDY}};
            Plan best;
            double best_ms = -1.0;
            int best_pol = -1;
            for (auto& c : cands) {
                compile_plan(n, c[0], c[1], p);
                if (!p.ok) continue;
                const double ms = estimate_step_ms(n, p);
                if (best_pol < 0 || ms < best_ms) { best = p; best_ms = ms; best_pol = c[0]; }
            }
            if (best_pol >= 0) { n.plan = best; n.policy = policy; n.effective = best_pol; return VDNN_OK; }
            n.plan = first; n.policy = policy; n.effective = VDNN_POLICY_ALL;
            return VDNN_OK;
        }
        const int order[3] = {VDNN_POLICY_NONE, VDNN_POLICY_CONV, VDNN_POLICY_ALL};
        for (int pol : order) {
            compile_plan(n, pol, VDNN_ALGO_PERF, p);
            if (p.ok) { n.plan = p; n.policy = policy; n.effective = pol; return VDNN_OK; }
        }
        for (int pol : {VDNN_POLICY_CONV, VDNN_POLICY_ALL}) {
            compile_plan(n, pol, VDNN_ALGO_GREEDY, p);
            if (p.ok) { n.plan = p; n.policy = policy; n.effective = pol; return VDNN_OK; }
        }
        n.plan = first; n.policy = policy; n.effective = VDNN_POLICY_ALL;
        return VDNN_OK;
    }
    compile_plan(n, policy, n.static_algo, p);
    if (!p.ok) { n.err = p.fail_why; return VDNN_ERR_OOM_DEVICE; }
    n.plan = p; n.policy = policy; n.effective = policy;
    return VDNN_OK;
}

}  // namespace vdnn
