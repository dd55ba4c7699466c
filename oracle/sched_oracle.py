"""Plain-Python oracle of the host-side memory scheduling of SuperNeurons (arXiv 1801.04380) --
TEST INFRASTRUCTURE, not part of the product.  Written from the paper's description with sets and
dictionaries, nothing tuned; it shares no code with the C++ implementation it checks
(csrc/sn_runtime.cpp), and only tests may import it.

What it models, in the paper's order:
  route(...)            Alg. 1: execution order of a nonlinear network (depth first, a join waits
                        for all of its inputs).
  Pool                  Sec. 3.2.1: heap memory pool in 1 KB blocks, first fit over the list of
                        empty nodes, deallocation by node id.
  memory_trace(...)     Sec. 3.2 (liveness analysis: a tensor is freed after the last step that
                        needs it), Sec. 3.3.1 (offloading / prefetching with the CONV outputs as
                        checkpoints), Sec. 3.4 (speed-centric, memory-centric and cost-aware
                        recomputation) -> bytes and live tensor count per step, extra forward
                        computations.  Sec. 4.1 and Table 1 print numbers for AlexNet at batch 200;
                        the tests pin this file to them.

Readings of the paper this file takes (each is listed in the design notes as well):
  * Steps are numbered as in Sec. 4.1: forward step s = s-th layer of the route after the data
    layer, backward steps follow in reverse order (N layers: steps 1..N and N+1..2N).
  * A layer's backward needs these forward tensors: CONV, FC: its input; ACT, LRN, POOL: input and
    output; BN: input; SOFTMAX: output; DROPOUT, JOIN: none.  The data tensor is needed by the
    forward of its consumers only (the numbers of Sec. 4.1 leave it out of every backward step).
  * Gradient tensors: a layer's backward writes the gradient of each of its inputs into a tensor
    of its own, except ACT, LRN (in place: the gradient of the input takes the place of the
    gradient of the output) and SOFTMAX (the gradient of its input takes the place of its own
    output); no gradient of the data.  This is the only assignment of tensors to layers that gives
    Sec. 4.1's 36 tensors / 2189.437 MB.
  * Offloading: a CONV output leaves the GPU once its forward consumers have run; in the backward
    it is on the GPU during the steps from the nearest CONV layer at or before the step, in route
    order, to the step itself, if one of them needs it (Sec. 3.3.1: a CONV layer's backward fetches
    what the steps down to the previous CONV layer need).
  * Recomputation: outputs of ACT, LRN, POOL, BN, DROPOUT are dropped after their forward
    consumers have run.  A segment is a maximal chain of such layers; its head is the kept tensor
    it starts from.  Speed-centric: the first backward step that needs a tensor of the segment
    recomputes the whole segment and keeps it.  Memory-centric: every backward step recomputes the
    chain up to the tensors it needs, dropping the intermediates as it goes and keeping what it
    asked for until its last use.  Cost-aware: l_peak is the peak of the memory-centric trace; a
    segment runs speed-centric iff its speed-centric steps stay within l_peak.
"""
BLOCK = 1024

DATA, CONV, ACT, LRN, POOL, BN, FC, DROPOUT, SOFTMAX, JOIN = range(10)
KIND_NAMES = ["DATA", "CONV", "ACT", "LRN", "POOL", "BN", "FC", "DROPOUT", "SOFTMAX", "JOIN"]
NEEDS_X = {CONV, FC, ACT, LRN, POOL, BN}
NEEDS_Y = {ACT, LRN, POOL, SOFTMAX}
INPLACE_BWD = {ACT, LRN}
RECOMPUTABLE = {ACT, LRN, POOL, BN, DROPOUT}

BASELINE, LIVENESS, OFFLOAD, RECOMPUTE = range(4)
SPEED, MEMORY, COST_AWARE = range(3)


class Net:
    """layers[i] = (kind, out_bytes, [ids of the layers whose outputs it reads])."""

    def __init__(self):
        self.layers = []

    def add(self, kind, out_bytes, prev=()):
        self.layers.append((kind, int(out_bytes), list(prev)))
        return len(self.layers) - 1

    def nexts(self, i):
        return [j for j, (_, _, prev) in enumerate(self.layers) if i in prev]


def route(net):
    """Alg. 1: starting at the data layer, visit depth first; a layer runs once all of the layers
    before it have run (a counter per layer), and the search goes on from it."""
    order, counter = [], [0] * len(net.layers)

    def construct(i):
        counter[i] += 1
        if counter[i] < len(net.layers[i][2]):
            return
        order.append(i)
        for j in net.nexts(i):
            construct(j)
        counter[i] = 0

    starts = [i for i, (k, _, prev) in enumerate(net.layers) if not prev]
    for s in starts:
        construct(s)
    return order


class Pool:
    """Sec. 3.2.1: the pool is cut into 1 KB blocks; an allocation takes the first empty node
    with enough blocks; a deallocation finds its node by id and puts it back among the empty
    ones (neighbouring empty nodes merge, which the paper does not spell out)."""

    def __init__(self, nbytes):
        self.nblocks = nbytes // BLOCK
        self.empty = [(0, self.nblocks)] if self.nblocks else []   # (first block, blocks), by address
        self.used = {}                                            # id -> (first block, blocks)
        self.next_id = 1
        self.used_blocks = 0
        self.peak_blocks = 0
        self.high_water = 0

    def alloc(self, nbytes):
        need = max(1, -(-nbytes // BLOCK))
        for n, (start, size) in enumerate(self.empty):
            if size >= need:
                if size == need:
                    del self.empty[n]
                else:
                    self.empty[n] = (start + need, size - need)
                ident = self.next_id
                self.next_id += 1
                self.used[ident] = (start, need)
                self.used_blocks += need
                self.peak_blocks = max(self.peak_blocks, self.used_blocks)
                self.high_water = max(self.high_water, start + need)
                return ident, start * BLOCK
        return None

    def free(self, ident):
        start, size = self.used.pop(ident)
        self.used_blocks -= size
        self.empty.append((start, size))
        self.empty.sort()
        merged = []
        for s, z in self.empty:
            if merged and merged[-1][0] + merged[-1][1] == s:
                merged[-1] = (merged[-1][0], merged[-1][1] + z)
            else:
                merged.append((s, z))
        self.empty = merged

    def largest_free(self):
        return max((z for _, z in self.empty), default=0) * BLOCK


def _analyse(net):
    """Route positions, consumers, gradient buffers (alias classes) and segments."""
    order = route(net)
    steps = [i for i in order if net.layers[i][0] != DATA]       # forward step s runs steps[s - 1]
    pos = {i: s + 1 for s, i in enumerate(steps)}                # layer -> forward step (data: none)
    cons = {i: net.nexts(i) for i in range(len(net.layers))}
    last = steps[-1]
    # gradient buffer of the output of layer i: grad[i] = name of the buffer, or None
    grad = {}
    for i in reversed(steps):
        kind = net.layers[i][0]
        if i == last or not cons[i]:
            grad[i] = None if kind == SOFTMAX or i == last else ("G", i)
            continue
        c = cons[i]
        only = c[0] if len(c) == 1 else None
        if only is not None and net.layers[only][0] in INPLACE_BWD and len(net.layers[only][2]) == 1 and grad[only]:
            grad[i] = grad[only]                                  # in place: takes over the output's gradient
        elif only is not None and net.layers[only][0] == SOFTMAX:
            grad[i] = ("F", only)                                 # written over the softmax output
        else:
            grad[i] = ("G", i)
    return order, steps, pos, cons, grad


def _bwd_needs(net, i):
    kind, _, prev = net.layers[i]
    need = set()
    if kind in NEEDS_X:
        need |= {j for j in prev if net.layers[j][0] != DATA}
    if kind in NEEDS_Y:
        need.add(i)
    return need


def memory_trace(net, level, strategy=COST_AWARE):
    """-> dict(bytes=[...], live=[...], peak, peak_step, extra, tensors) over steps 1..2N
    (index s - 1); bytes[s - 1] is the most that is allocated at any moment of step s."""
    order, steps, pos, cons, grad = _analyse(net)
    N = len(steps)
    size = {("F", i): net.layers[i][1] for i in range(len(net.layers))}
    for i in steps:
        if grad[i] and grad[i][0] == "G":
            size[grad[i]] = net.layers[i][1]
    if level == BASELINE:
        total = sum(size.values())
        return dict(bytes=[total] * (2 * N), live=[len(size)] * (2 * N), peak=total, peak_step=1, extra=0,
                    tensors=len(size))

    def bstep(i):
        return 2 * N + 1 - pos[i]

    data_ids = [i for i in range(len(net.layers)) if net.layers[i][0] == DATA]
    # ---- every use of every tensor: (step, tensor)
    fwd_use, bwd_use = {}, {}
    for i in steps:
        for j in net.layers[i][2]:
            fwd_use.setdefault(("F", j), []).append(pos[i])
        fwd_use.setdefault(("F", i), []).append(pos[i])
        for j in _bwd_needs(net, i):
            bwd_use.setdefault(("F", j), []).append(bstep(i))
    for i in steps:
        g = grad[i]
        if g:
            bwd_use.setdefault(g, []).append(bstep(i))             # read as the gradient of the output
            for c in cons[i]:
                bwd_use.setdefault(g, []).append(bstep(c))         # written by the consumers' backward
    conv_pos = sorted(pos[i] for i in steps if net.layers[i][0] == CONV)

    def prev_conv_step(s):
        """Backward step of the nearest CONV layer at or before the layer of backward step s."""
        p = 2 * N + 1 - s
        at = [c for c in conv_pos if c <= p]
        return 2 * N + 1 - (at[-1] if at else 1)

    dropped = set()      # forward tensors that leave the GPU after their forward uses
    if level >= OFFLOAD:
        dropped |= {("F", i) for i in steps if net.layers[i][0] == CONV}
    recomp = set()
    if level >= RECOMPUTE:
        recomp = {("F", i) for i in steps if net.layers[i][0] in RECOMPUTABLE}
        dropped |= recomp

    def head_chain(t):
        """The recomputable tensors to produce, in order, to get t, and the kept tensors they start from."""
        chain, heads, seen = [], set(), set()

        def visit(u):
            if u in seen:
                return
            seen.add(u)
            if u not in recomp:
                heads.add(u)
                return
            for j in net.layers[u[1]][2]:
                visit(("F", j))
            chain.append(u)

        visit(t)
        return chain, heads

    def segment_of(t):
        """All recomputable tensors connected to t through recomputable producers / consumers."""
        seg, todo = set(), [t]
        while todo:
            u = todo.pop()
            if u in seg or u not in recomp:
                continue
            seg.add(u)
            todo += [("F", j) for j in net.layers[u[1]][2]] + [("F", c) for c in cons[u[1]]]
        return seg

    def wanted_at(s):
        """Offloaded checkpoints on the GPU during backward step s: those that a step from s down to
        the backward of the nearest CONV layer at or before it needs, directly or as the tensor a
        recomputation starts from."""
        out = set()
        for s2 in range(s, prev_conv_step(s) + 1):
            for j in _bwd_needs(net, steps[2 * N - s2]):
                t = ("F", j)
                for u in (head_chain(t)[1] if t in recomp else {t}):
                    if u in dropped and u not in recomp:
                        out.add(u)
        return out

    def run(seg_strategy):
        """One pass over the 2N steps.  seg_strategy(frozenset segment) -> SPEED or MEMORY."""
        live = {}
        out_b, out_n = [0] * (2 * N), [0] * (2 * N)
        extra = [0]
        cur = [0]

        def alloc(t, s):
            if t not in live:
                live[t] = True
                cur[0] += size[t]
                out_b[s - 1] = max(out_b[s - 1], cur[0])
                out_n[s - 1] = max(out_n[s - 1], len(live))

        def release(t):
            if t in live:
                del live[t]
                cur[0] -= size[t]

        def last_use(t):
            return max(fwd_use.get(t, [0]) + bwd_use.get(t, [0]))

        for d in data_ids:
            live[("F", d)] = True
            cur[0] += size[("F", d)]
        for s in range(1, N + 1):                                   # forward
            i = steps[s - 1]
            out_b[s - 1], out_n[s - 1] = cur[0], len(live)
            alloc(("F", i), s)
            for t in list(live):
                if max(fwd_use.get(t, [0])) <= s and (t in dropped or not bwd_use.get(t)):
                    release(t)
        for s in range(N + 1, 2 * N + 1):                           # backward
            i = steps[2 * N - s]
            out_b[s - 1], out_n[s - 1] = cur[0], len(live)
            for t in wanted_at(s):
                alloc(t, s)
            # recomputation of what this step needs
            for t in sorted(("F", j) for j in _bwd_needs(net, i)):
                if t not in recomp or t in live:
                    continue
                seg = frozenset(segment_of(t))
                if seg_strategy(seg) == SPEED:
                    members = sorted(seg, key=lambda u: pos[u[1]])
                    for u in members:
                        if u not in live:
                            for h in head_chain(u)[1]:
                                alloc(h, s)
                            alloc(u, s)
                            extra[0] += 1
                else:
                    chain, heads = head_chain(t)
                    for h in heads:
                        alloc(h, s)
                    made = []
                    for u in chain:
                        if u in live:
                            continue
                        alloc(u, s)
                        extra[0] += 1
                        made.append(u)
                        # intermediates go as soon as everything made from them in this chain exists
                        for v in list(made):
                            if v != t and v not in {("F", j) for j in _bwd_needs(net, i)}:
                                users = [w for w in chain if v[1] in net.layers[w[1]][2]]
                                if all(w in live for w in users):
                                    release(v)
                                    made.remove(v)
            g_in = grad[i]
            if g_in:
                alloc(g_in, s)                                      # exists already unless this is the last layer
            for j in net.layers[i][2]:
                if net.layers[j][0] != DATA and grad[j]:
                    alloc(grad[j], s)
            nxt = wanted_at(s + 1) if s < 2 * N else set()
            for t in list(live):
                if t in dropped and t not in recomp:
                    if t not in nxt:
                        release(t)                                  # a fetched checkpoint nobody down to the previous CONV needs
                elif last_use(t) <= s:
                    release(t)
        peak = max(out_b)
        return dict(bytes=out_b, live=out_n, peak=peak, peak_step=out_b.index(peak) + 1, extra=extra[0],
                    tensors=len(size))

    if level < RECOMPUTE or strategy == SPEED:
        return run(lambda seg: SPEED)
    mem = run(lambda seg: MEMORY)
    if strategy == MEMORY:
        return mem
    # cost-aware: a segment runs speed-centric iff its steps then stay within the memory-centric peak
    spd = run(lambda seg: SPEED)
    l_peak = mem["peak"]
    choice = {}
    for i in steps:
        t = ("F", i)
        if t in recomp:
            seg = frozenset(segment_of(t))
            if seg not in choice:
                first = min(pos[u[1]] for u in seg)
                lastp = max(pos[u[1]] for u in seg)
                trigger = min([bstep(c) for u in seg for c in cons[u[1]] if ("F", c) not in seg] + [bstep(steps[lastp - 1])])
                span = range(trigger, bstep(steps[first - 1]) + 1)
                choice[seg] = SPEED if max(spd["bytes"][s - 1] for s in span) <= l_peak else MEMORY
    res = run(lambda seg: choice[seg])
    res["l_peak"] = l_peak
    return res


def alexnet(batch=200, elem=4):
    """The AlexNet of Sec. 4.1 (footnote: CONV1 RELU1 LRN1 POOL1 CONV2 RELU2 LRN2 POOL2 CONV3 RELU3
    CONV4 RELU4 CONV5 RELU5 POOL5 FC1 RELU6 Dropout1 FC2 RELU7 Dropout2 FC3 Softmax), tensor sizes
    from its 227 x 227 input: 96@55x55, 256@27x27, 384@13x13 (the paper prints the first three)."""
    net = Net()
    b = batch * elem
    prev = net.add(DATA, b * 3 * 227 * 227)
    spec = [(CONV, 96 * 55 * 55), (ACT, 96 * 55 * 55), (LRN, 96 * 55 * 55), (POOL, 96 * 27 * 27),
            (CONV, 256 * 27 * 27), (ACT, 256 * 27 * 27), (LRN, 256 * 27 * 27), (POOL, 256 * 13 * 13),
            (CONV, 384 * 13 * 13), (ACT, 384 * 13 * 13), (CONV, 384 * 13 * 13), (ACT, 384 * 13 * 13),
            (CONV, 256 * 13 * 13), (ACT, 256 * 13 * 13), (POOL, 256 * 6 * 6),
            (FC, 4096), (ACT, 4096), (DROPOUT, 4096), (FC, 4096), (ACT, 4096), (DROPOUT, 4096),
            (FC, 1000), (SOFTMAX, 1000)]
    for kind, elems in spec:
        prev = net.add(kind, b * elems, [prev])
    return net
