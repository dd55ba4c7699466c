// Host side of sn_runtime.h: the memory pool of Sec. 3.2.1, the execution order of Alg. 1, and
// the step-by-step memory model of Liveness Analysis (Sec. 3.2), Offloading / Prefetching
// (Sec. 3.3.1) and Recomputation (Sec. 3.4) that yields the per-step workspace budgets of
// Sec. 3.5.  Sizes and step numbers only: no device memory, no launches.
#include <algorithm>
#include <cstdint>
#include <cstring>
#include <list>
#include <map>
#include <new>
#include <unordered_map>
#include <vector>

#include "sn_runtime.h"

// ---- memory pool ------------------------------------------------------------------------------
// Two lists of nodes as in the paper: the empty nodes ordered by address (so that "the first node
// with enough free memory" is also the lowest one and neighbours can merge), and the allocated
// nodes reached through an id -> node hash table.
struct sn_pool {
    struct Node { size_t first, blocks; };
    std::list<Node> empty;
    std::unordered_map<uint64_t, Node> allocated;
    uint64_t next_id = 1;
    size_t total = 0, used = 0, peak = 0, high = 0;
};

extern "C" {

sn_pool *sn_pool_create(size_t bytes)
{
    sn_pool *p = new (std::nothrow) sn_pool;
    if (!p) return nullptr;
    p->total = bytes / SN_POOL_BLOCK;
    if (p->total) p->empty.push_back({0, p->total});
    return p;
}

void sn_pool_destroy(sn_pool *pool) { delete pool; }

sn_status sn_pool_alloc(sn_pool *pool, size_t bytes, uint64_t *id, size_t *offset)
{
    if (!pool || !id || !offset) return SN_ERR_BAD_ARG;
    const size_t need = bytes ? (bytes + SN_POOL_BLOCK - 1) / SN_POOL_BLOCK : 1;
    for (auto it = pool->empty.begin(); it != pool->empty.end(); ++it) {
        if (it->blocks < need) continue;
        const sn_pool::Node got = {it->first, need};
        if (it->blocks == need) pool->empty.erase(it);
        else { it->first += need; it->blocks -= need; }
        *id = pool->next_id++;
        pool->allocated.emplace(*id, got);
        pool->used += need;
        pool->peak = std::max(pool->peak, pool->used);
        pool->high = std::max(pool->high, got.first + need);
        *offset = got.first * SN_POOL_BLOCK;
        return SN_OK;
    }
    return SN_ERR_WORKSPACE_TOO_SMALL;
}

sn_status sn_pool_free(sn_pool *pool, uint64_t id)
{
    if (!pool) return SN_ERR_BAD_ARG;
    auto f = pool->allocated.find(id);
    if (f == pool->allocated.end()) return SN_ERR_BAD_ARG;
    sn_pool::Node n = f->second;
    pool->allocated.erase(f);
    pool->used -= n.blocks;
    // insert by address, then merge with the node before and the node after
    auto at = pool->empty.begin();
    while (at != pool->empty.end() && at->first < n.first) ++at;
    at = pool->empty.insert(at, n);
    auto nx = std::next(at);
    if (nx != pool->empty.end() && at->first + at->blocks == nx->first) {
        at->blocks += nx->blocks;
        pool->empty.erase(nx);
    }
    if (at != pool->empty.begin()) {
        auto pv = std::prev(at);
        if (pv->first + pv->blocks == at->first) {
            pv->blocks += at->blocks;
            pool->empty.erase(at);
        }
    }
    return SN_OK;
}

size_t sn_pool_used_bytes(const sn_pool *pool) { return pool ? pool->used * SN_POOL_BLOCK : 0; }
size_t sn_pool_peak_bytes(const sn_pool *pool) { return pool ? pool->peak * SN_POOL_BLOCK : 0; }
size_t sn_pool_high_water(const sn_pool *pool) { return pool ? pool->high * SN_POOL_BLOCK : 0; }

size_t sn_pool_largest_free(const sn_pool *pool)
{
    size_t best = 0;
    if (pool)
        for (const auto &n : pool->empty) best = std::max(best, n.blocks);
    return best * SN_POOL_BLOCK;
}

}  // extern "C"

// ---- network ------------------------------------------------------------------------------------
struct sn_net {
    struct Layer {
        int kind;
        size_t bytes;
        std::vector<int> prev, next;
        bool has_shape = false;
        sn_conv_shape shape;
    };
    std::vector<Layer> layers;
};

namespace {

bool needs_input(int kind) { return kind == SN_L_CONV || kind == SN_L_FC || kind == SN_L_ACT || kind == SN_L_LRN || kind == SN_L_POOL || kind == SN_L_BN; }
bool needs_output(int kind) { return kind == SN_L_ACT || kind == SN_L_LRN || kind == SN_L_POOL || kind == SN_L_SOFTMAX; }
bool backward_in_place(int kind) { return kind == SN_L_ACT || kind == SN_L_LRN; }
bool cheap(int kind) { return kind == SN_L_ACT || kind == SN_L_LRN || kind == SN_L_POOL || kind == SN_L_BN || kind == SN_L_DROPOUT; }

// Alg. 1 with an explicit stack: a layer runs when its counter reaches the number of its inputs,
// then its successors are visited in the order they were added.
std::vector<int> execution_order(const sn_net &net)
{
    const int L = (int)net.layers.size();
    std::vector<int> order, counter(L, 0);
    struct Frame { int layer; size_t child; };
    for (int start = 0; start < L; ++start) {
        if (!net.layers[start].prev.empty()) continue;
        std::vector<Frame> stack;
        order.push_back(start);
        stack.push_back({start, 0});
        while (!stack.empty()) {
            Frame &f = stack.back();
            const auto &nx = net.layers[f.layer].next;
            if (f.child == nx.size()) {
                counter[f.layer] = 0;
                stack.pop_back();
                continue;
            }
            const int c = nx[f.child++];
            if (++counter[c] < (int)net.layers[c].prev.size()) continue;   // a join still waiting
            order.push_back(c);
            stack.push_back({c, 0});
        }
    }
    return order;
}

// Everything the step simulation needs to know about the network, worked out once per call.
struct Model {
    const sn_net &net;
    int L, N;                          // layers, steps per direction
    std::vector<int> at;               // forward step s (1-based) runs layer at[s]
    std::vector<int> fstep;            // layer -> forward step, 0 for data / unreachable layers
    // tensors: 0 .. L-1 forward outputs, L .. gradient tensors
    std::vector<size_t> bytes;
    std::vector<int> grad;             // layer -> tensor holding the gradient of its output, -1 none
    std::vector<int> last_use;         // tensor -> last step that touches it
    std::vector<int> last_fwd_use;
    std::vector<char> used_in_bwd;
    std::vector<std::vector<int>> need;   // backward needs of a layer: forward tensors
    std::vector<char> offloaded, dropped_cheap;
    std::vector<int> conv_steps;       // forward steps of the CONV layers, ascending
    int ntensors_baseline = 0;

    explicit Model(const sn_net &n) : net(n)
    {
        L = (int)net.layers.size();
        const std::vector<int> order = execution_order(net);
        at.push_back(-1);
        fstep.assign(L, 0);
        for (int id : order)
            if (net.layers[id].kind != SN_L_DATA) {
                fstep[id] = (int)at.size();
                at.push_back(id);
            }
        N = (int)at.size() - 1;
        bytes.resize(L);
        for (int i = 0; i < L; ++i) bytes[i] = net.layers[i].bytes;
        // gradient tensors, from the last layer backwards so that an in-place layer finds the
        // tensor of its output's gradient
        grad.assign(L, -1);
        for (int s = N; s >= 1; --s) {
            const int i = at[s];
            std::vector<int> users;
            for (int c : net.layers[i].next)
                if (fstep[c]) users.push_back(c);
            if (s == N || users.empty()) {
                if (s != N && net.layers[i].kind != SN_L_SOFTMAX) grad[i] = new_tensor(bytes[i]);
                continue;
            }
            const int only = users.size() == 1 ? users[0] : -1;
            if (only >= 0 && backward_in_place(net.layers[only].kind) && net.layers[only].prev.size() == 1 && grad[only] >= 0)
                grad[i] = grad[only];
            else if (only >= 0 && net.layers[only].kind == SN_L_SOFTMAX)
                grad[i] = only;          // written over the softmax output
            else
                grad[i] = new_tensor(bytes[i]);
        }
        const int T = (int)bytes.size();
        ntensors_baseline = 0;
        for (int i = 0; i < L; ++i)
            if (fstep[i] || net.layers[i].kind == SN_L_DATA) ++ntensors_baseline;
        ntensors_baseline += T - L;
        // uses
        need.assign(L, {});
        last_use.assign(T, 0);
        last_fwd_use.assign(T, 0);
        used_in_bwd.assign(T, 0);
        for (int s = 1; s <= N; ++s) {
            const int i = at[s];
            const int kind = net.layers[i].kind;
            for (int j : net.layers[i].prev) last_fwd_use[j] = std::max(last_fwd_use[j], s);
            last_fwd_use[i] = std::max(last_fwd_use[i], s);
            const int b = bstep(i);
            if (needs_input(kind))
                for (int j : net.layers[i].prev)
                    if (net.layers[j].kind != SN_L_DATA) need[i].push_back(j);
            if (needs_output(kind)) need[i].push_back(i);
            std::sort(need[i].begin(), need[i].end());
            need[i].erase(std::unique(need[i].begin(), need[i].end()), need[i].end());
            for (int t : need[i]) { last_use[t] = std::max(last_use[t], b); used_in_bwd[t] = 1; }
            if (grad[i] >= 0) {
                last_use[grad[i]] = std::max(last_use[grad[i]], b);
                used_in_bwd[grad[i]] = 1;
            }
            for (int j : net.layers[i].prev)
                if (net.layers[j].kind != SN_L_DATA && grad[j] >= 0) {
                    last_use[grad[j]] = std::max(last_use[grad[j]], b);
                    used_in_bwd[grad[j]] = 1;
                }
            if (kind == SN_L_CONV) conv_steps.push_back(s);
        }
        for (int t = 0; t < T; ++t) last_use[t] = std::max(last_use[t], last_fwd_use[t]);
    }

    int new_tensor(size_t b) { bytes.push_back(b); return (int)bytes.size() - 1; }
    int bstep(int layer) const { return 2 * N + 1 - fstep[layer]; }
    int layer_of_step(int s) const { return s <= N ? at[s] : at[2 * N + 1 - s]; }

    // Backward step of the nearest CONV layer at or before the layer of backward step s.
    int conv_horizon(int s) const
    {
        const int p = 2 * N + 1 - s;
        auto it = std::upper_bound(conv_steps.begin(), conv_steps.end(), p);
        const int c = it == conv_steps.begin() ? 1 : *(it - 1);
        return 2 * N + 1 - c;
    }
};

// One pass over the iteration under a given level and per-segment strategy.
struct Simulation {
    const Model &m;
    int level;
    std::vector<char> live;
    std::vector<char> cheap_t, ckpt_t;      // forward tensor is recomputed / offloaded
    std::vector<int> segment;               // forward tensor -> segment number, -1
    int nsegments = 0;
    std::vector<int> seg_strategy;          // per segment
    size_t cur = 0;
    int nlive = 0;
    std::vector<size_t> step_bytes;
    std::vector<int> step_live;
    int extra = 0;
    int step = 0;

    Simulation(const Model &model, int lvl) : m(model), level(lvl)
    {
        const int T = (int)m.bytes.size();
        live.assign(T, 0);
        cheap_t.assign(T, 0);
        ckpt_t.assign(T, 0);
        segment.assign(T, -1);
        for (int s = 1; s <= m.N; ++s) {
            const int i = m.at[s], kind = m.net.layers[i].kind;
            if (level >= SN_MEM_OFFLOAD && kind == SN_L_CONV) ckpt_t[i] = 1;
            if (level >= SN_MEM_RECOMPUTE && cheap(kind)) cheap_t[i] = 1;
        }
        // segments: connected sets of recomputed tensors (through producer / consumer links)
        for (int s = 1; s <= m.N; ++s) {
            const int i = m.at[s];
            if (!cheap_t[i] || segment[i] >= 0) continue;
            std::vector<int> todo{i};
            while (!todo.empty()) {
                const int u = todo.back();
                todo.pop_back();
                if (!cheap_t[u] || segment[u] >= 0) continue;
                segment[u] = nsegments;
                for (int j : m.net.layers[u].prev) todo.push_back(j);
                for (int c : m.net.layers[u].next)
                    if (m.fstep[c]) todo.push_back(c);
            }
            ++nsegments;
        }
        seg_strategy.assign(nsegments, SN_RECOMP_SPEED);
        step_bytes.assign(2 * m.N, 0);
        step_live.assign(2 * m.N, 0);
    }

    void hold(int t)
    {
        if (live[t]) return;
        live[t] = 1;
        cur += m.bytes[t];
        ++nlive;
        step_bytes[step - 1] = std::max(step_bytes[step - 1], cur);
        step_live[step - 1] = std::max(step_live[step - 1], nlive);
    }
    void drop(int t)
    {
        if (!live[t]) return;
        live[t] = 0;
        cur -= m.bytes[t];
        --nlive;
    }

    // The kept tensors a recomputation of forward tensor t starts from, and (optionally) the cheap
    // tensors to produce on the way, producers before consumers.
    void sources(int t, std::vector<int> *heads, std::vector<int> *chain, std::vector<char> &seen) const
    {
        if (seen[t]) return;
        seen[t] = 1;
        if (!cheap_t[t]) {
            heads->push_back(t);
            return;
        }
        for (int j : m.net.layers[t].prev) sources(j, heads, chain, seen);
        if (chain) chain->push_back(t);
    }

    // Offloaded checkpoints that are on the GPU during backward step s.
    std::vector<int> fetched_at(int s) const
    {
        std::vector<int> out;
        std::vector<char> seen(m.L, 0);
        for (int s2 = s; s2 <= m.conv_horizon(s); ++s2)
            for (int t : m.need[m.layer_of_step(s2)]) {
                std::vector<int> heads;
                if (cheap_t[t]) sources(t, &heads, nullptr, seen);
                else if (!seen[t]) { seen[t] = 1; heads.push_back(t); }
                for (int h : heads)
                    if (ckpt_t[h]) out.push_back(h);
            }
        return out;
    }

    void recompute_for(int layer)
    {
        for (int t : m.need[layer]) {
            if (!cheap_t[t] || live[t]) continue;
            if (seg_strategy[segment[t]] == SN_RECOMP_SPEED) {
                // the whole segment, in execution order, and it stays
                for (int s = 1; s <= m.N; ++s) {
                    const int u = m.at[s];
                    if (segment[u] != segment[t] || live[u]) continue;
                    std::vector<int> heads;
                    std::vector<char> seen(m.L, 0);
                    sources(u, &heads, nullptr, seen);
                    for (int h : heads) hold(h);
                    hold(u);
                    ++extra;
                }
            } else {
                std::vector<int> heads, chain;
                std::vector<char> seen(m.L, 0);
                sources(t, &heads, &chain, seen);
                for (int h : heads) hold(h);
                std::vector<int> made;
                for (int u : chain) {
                    if (live[u]) continue;
                    hold(u);
                    ++extra;
                    made.push_back(u);
                    // an intermediate goes once everything made from it in this chain exists
                    for (size_t k = 0; k < made.size();) {
                        const int v = made[k];
                        bool asked = v == t || std::binary_search(m.need[layer].begin(), m.need[layer].end(), v);
                        bool done = true;
                        for (int w : chain)
                            if (std::find(m.net.layers[w].prev.begin(), m.net.layers[w].prev.end(), v) != m.net.layers[w].prev.end() && !live[w])
                                done = false;
                        if (!asked && done) {
                            drop(v);
                            made.erase(made.begin() + k);
                        } else {
                            ++k;
                        }
                    }
                }
            }
        }
    }

    void run()
    {
        for (int i = 0; i < m.L; ++i)
            if (m.net.layers[i].kind == SN_L_DATA) { live[i] = 1; cur += m.bytes[i]; ++nlive; }
        const int T = (int)m.bytes.size();
        for (step = 1; step <= m.N; ++step) {
            step_bytes[step - 1] = cur;
            step_live[step - 1] = nlive;
            hold(m.at[step]);
            for (int t = 0; t < T; ++t)
                if (live[t] && m.last_fwd_use[t] <= step && (ckpt_t[t] || cheap_t[t] || !m.used_in_bwd[t])) drop(t);
        }
        for (step = m.N + 1; step <= 2 * m.N; ++step) {
            const int layer = m.layer_of_step(step);
            step_bytes[step - 1] = cur;
            step_live[step - 1] = nlive;
            for (int t : fetched_at(step)) hold(t);
            recompute_for(layer);
            if (m.grad[layer] >= 0) hold(m.grad[layer]);
            for (int j : m.net.layers[layer].prev)
                if (m.net.layers[j].kind != SN_L_DATA && m.grad[j] >= 0) hold(m.grad[j]);
            std::vector<char> wanted(T, 0);
            if (step < 2 * m.N)
                for (int t : fetched_at(step + 1)) wanted[t] = 1;
            for (int t = 0; t < T; ++t) {
                if (!live[t]) continue;
                if (t < m.L && ckpt_t[t]) {
                    if (!wanted[t]) drop(t);
                } else if (m.last_use[t] <= step) {
                    drop(t);
                }
            }
        }
    }
};

struct Trace {
    std::vector<size_t> bytes;
    std::vector<int> live;
    sn_mem_summary sum;
};

void summarise(Trace &tr)
{
    tr.sum.peak_bytes = 0;
    tr.sum.peak_step = 1;
    for (size_t s = 0; s < tr.bytes.size(); ++s)
        if (tr.bytes[s] > tr.sum.peak_bytes) { tr.sum.peak_bytes = tr.bytes[s]; tr.sum.peak_step = (int)s + 1; }
}

Trace make_trace(const Model &m, int level, int strategy)
{
    Trace tr;
    std::memset(&tr.sum, 0, sizeof(tr.sum));
    tr.sum.tensors = m.ntensors_baseline;
    if (level == SN_MEM_BASELINE) {
        size_t total = 0;
        for (int t = 0; t < (int)m.bytes.size(); ++t)
            if (t >= m.L || m.fstep[t] || m.net.layers[t].kind == SN_L_DATA) total += m.bytes[t];
        tr.bytes.assign(2 * m.N, total);
        tr.live.assign(2 * m.N, m.ntensors_baseline);
        summarise(tr);
        return tr;
    }
    auto pass = [&](const std::vector<int> *choice, int uniform) {
        Simulation sim(m, level);
        for (int g = 0; g < sim.nsegments; ++g) sim.seg_strategy[g] = choice ? (*choice)[g] : uniform;
        sim.run();
        Trace t;
        std::memset(&t.sum, 0, sizeof(t.sum));
        t.bytes = sim.step_bytes;
        t.live = sim.step_live;
        t.sum.tensors = m.ntensors_baseline;
        t.sum.extra_forward = sim.extra;
        summarise(t);
        return t;
    };
    if (level < SN_MEM_RECOMPUTE || strategy == SN_RECOMP_SPEED) return pass(nullptr, SN_RECOMP_SPEED);
    Trace mem = pass(nullptr, SN_RECOMP_MEMORY);
    mem.sum.l_peak = mem.sum.peak_bytes;
    if (strategy == SN_RECOMP_MEMORY) return mem;
    // cost-aware: a segment runs speed-centric iff its steps then stay within the memory-centric peak
    const Trace spd = pass(nullptr, SN_RECOMP_SPEED);
    Simulation probe(m, level);
    std::vector<int> choice(probe.nsegments, SN_RECOMP_SPEED);
    for (int g = 0; g < probe.nsegments; ++g) {
        int first = m.N + 1, last = 0, trigger = 2 * m.N + 1;
        for (int s = 1; s <= m.N; ++s) {
            const int u = m.at[s];
            if (probe.segment[u] != g) continue;
            first = std::min(first, s);
            last = std::max(last, s);
            for (int c : m.net.layers[u].next)
                if (m.fstep[c] && probe.segment[c] != g) trigger = std::min(trigger, m.bstep(c));
        }
        trigger = std::min(trigger, 2 * m.N + 1 - last);
        size_t worst = 0;
        for (int s = trigger; s <= 2 * m.N + 1 - first; ++s) worst = std::max(worst, spd.bytes[s - 1]);
        choice[g] = worst <= mem.sum.peak_bytes ? SN_RECOMP_SPEED : SN_RECOMP_MEMORY;
    }
    Trace out = pass(&choice, 0);
    out.sum.l_peak = mem.sum.peak_bytes;
    return out;
}

bool valid_level(int l) { return l >= SN_MEM_BASELINE && l <= SN_MEM_RECOMPUTE; }
bool valid_strategy(int s) { return s >= SN_RECOMP_SPEED && s <= SN_RECOMP_COST_AWARE; }

}  // namespace

extern "C" {

sn_net *sn_net_create(void) { return new (std::nothrow) sn_net; }
void sn_net_destroy(sn_net *net) { delete net; }

int sn_net_add_layer(sn_net *net, sn_layer_kind kind, size_t out_bytes, const int *prev, int nprev)
{
    if (!net || kind < 0 || kind >= SN_L_KINDS || nprev < 0 || (nprev > 0 && !prev)) return -1;
    if ((kind == SN_L_DATA) != (nprev == 0)) return -1;
    const int id = (int)net->layers.size();
    for (int i = 0; i < nprev; ++i)
        if (prev[i] < 0 || prev[i] >= id) return -1;
    sn_net::Layer l;
    l.kind = kind;
    l.bytes = out_bytes;
    l.prev.assign(prev, prev + nprev);
    net->layers.push_back(l);
    for (int i = 0; i < nprev; ++i) {
        auto &nx = net->layers[prev[i]].next;
        if (std::find(nx.begin(), nx.end(), id) == nx.end()) nx.push_back(id);
    }
    return id;
}

sn_status sn_net_set_conv_shape(sn_net *net, int layer, const sn_conv_shape *shape)
{
    if (!net || !shape || layer < 0 || layer >= (int)net->layers.size()) return SN_ERR_BAD_ARG;
    if (net->layers[layer].kind != SN_L_CONV) return SN_ERR_BAD_ARG;
    net->layers[layer].shape = *shape;
    net->layers[layer].has_shape = true;
    return SN_OK;
}

int sn_net_layers(const sn_net *net) { return net ? (int)net->layers.size() : 0; }

int sn_net_route(const sn_net *net, int *route, int cap)
{
    if (!net || (!route && cap > 0)) return -1;
    const std::vector<int> order = execution_order(*net);
    if ((int)order.size() > cap) return -1;
    std::copy(order.begin(), order.end(), route);
    return (int)order.size();
}

int sn_net_steps(const sn_net *net)
{
    if (!net) return 0;
    Model m(*net);
    return 2 * m.N;
}

sn_status sn_net_memory_trace(const sn_net *net, sn_mem_level level, sn_recomp_strategy strategy,
                              size_t *bytes_per_step, int32_t *live_per_step, sn_mem_summary *summary)
{
    if (!net || !valid_level(level) || !valid_strategy(strategy)) return SN_ERR_BAD_ARG;
    Model m(*net);
    if (m.N < 1) return SN_ERR_BAD_ARG;
    const Trace tr = make_trace(m, level, strategy);
    if (bytes_per_step) std::copy(tr.bytes.begin(), tr.bytes.end(), bytes_per_step);
    if (live_per_step) std::copy(tr.live.begin(), tr.live.end(), live_per_step);
    if (summary) *summary = tr.sum;
    return SN_OK;
}

sn_status sn_net_step_budgets(const sn_net *net, sn_mem_level level, sn_recomp_strategy strategy,
                              size_t capacity_bytes, size_t *free_per_step)
{
    if (!net || !free_per_step || !valid_level(level) || !valid_strategy(strategy)) return SN_ERR_BAD_ARG;
    Model m(*net);
    if (m.N < 1) return SN_ERR_BAD_ARG;
    const Trace tr = make_trace(m, level, strategy);
    for (size_t s = 0; s < tr.bytes.size(); ++s)
        free_per_step[s] = capacity_bytes > tr.bytes[s] ? capacity_bytes - tr.bytes[s] : 0;
    return SN_OK;
}

int sn_net_plan_convs(const sn_net *net, sn_mem_level level, sn_recomp_strategy strategy, size_t capacity_bytes,
                      sn_conv_step_plan *plans, int cap)
{
    if (!net || !valid_level(level) || !valid_strategy(strategy) || (!plans && cap > 0)) return -1;
    Model m(*net);
    if (m.N < 1) return -1;
    const Trace tr = make_trace(m, level, strategy);
    int n = 0;
    for (int s = 1; s <= m.N; ++s) {
        const int id = m.at[s];
        const sn_net::Layer &l = net->layers[id];
        if (l.kind != SN_L_CONV || !l.has_shape) continue;
        if (n >= cap) return -1;
        sn_conv_step_plan p;
        std::memset(&p, 0, sizeof(p));
        p.layer = id;
        p.fwd_step = s;
        p.bwd_step = 2 * m.N + 1 - s;
        // the workspace is carved from the pool in 256-byte units (the alignment the CONV calls ask for)
        auto room = [&](int step) {
            const size_t used = tr.bytes[step - 1];
            return capacity_bytes > used ? (capacity_bytes - used) / 256 * 256 : (size_t)0;
        };
        p.fwd_budget = room(p.fwd_step);
        p.bwd_budget = room(p.bwd_step);
        sn_conv_algo a;
        size_t ws;
        if (sn_conv_plan(&l.shape, SN_CONV_FWD, p.fwd_budget, &a, &ws, nullptr) != SN_OK) return -1;
        p.algo_fwd = a; p.ws_fwd = ws;
        if (sn_conv_plan(&l.shape, SN_CONV_BWD_DATA, p.bwd_budget, &a, &ws, nullptr) != SN_OK) return -1;
        p.algo_bwd_data = a; p.ws_bwd_data = ws;
        if (sn_conv_plan(&l.shape, SN_CONV_BWD_FILTER, p.bwd_budget, &a, &ws, nullptr) != SN_OK) return -1;
        p.algo_bwd_filter = a; p.ws_bwd_filter = ws;
        plans[n++] = p;
    }
    return n;
}

}  // extern "C"
