"""CPU oracle of the paper's planning steps (test infrastructure only: tests import it, the
product never does).  Plain Python, integers only.

  * k-way transmission order: Section 4.2, Algorithm 1.
  * sub-group sizes for k -> N scaling: Section 4.2, "Multicast and sub-groups".
  * execution pipeline generation: Section 4.3, Algorithm 2.
  * number of multicast steps of the binomial pipeline: Section 4.2 (b + ceil(log2 N) - 1).
  * a step-by-step schedule of that multicast for N = 2^n nodes.  The paper only cites the
    technique and states its step count; the schedule here is a construction of this build
    (exchange partners walk the hypercube dimensions, every node forwards its newest useful
    block) that meets the stated count.

Reading taken where the text is garbled: the sentence on sub-group sizes gives "floor(N/k) or
N%k"; a remainder is not a size, so the N nodes are dealt out as evenly as possible: the
first N mod k sub-groups hold ceil(N/k) nodes, the others floor(N/k).
"""


def chunk_span(b, k, i):
    """Blocks [lo, hi) of chunk i when b ordered blocks are cut into k chunks of ceil(b/k)."""
    size = -(-b // k)
    return min(size * i, b), min(size * (i + 1), b)


def kway_order(b, k, group):
    """Order in which sub-group `group` receives the b blocks: the chunks, starting with
    the group's own and wrapping around."""
    order = []
    for j in range(k):
        lo, hi = chunk_span(b, k, (group + j) % k)
        order.extend(range(lo, hi))
    return order


def subgroup_sizes(n_nodes, k):
    base, extra = divmod(n_nodes, k)
    return [base + (1 if i < extra else 0) for i in range(k)]


def pipelines(sizes):
    """sizes[i] = nodes of sub-group i that can join a pipeline.  Returns the pipelines in
    the order they are formed, each a list of (sub-group, node index inside it).

    Stated by depth instead of by rounds: a pipeline takes one node from every sub-group that
    still has one, and nodes join in index order, so the t-th pipeline is made of the t-th
    node of every sub-group holding more than t nodes -- as long as at least two sub-groups
    reach that depth.  Beyond it at most one sub-group has nodes left, and those form one
    last pipeline among themselves."""
    def at_depth(t):
        return [(i, t) for i, n in enumerate(sizes) if n > t]

    out, t = [], 0
    while len(at_depth(t)) >= 2:
        out.append(at_depth(t))
        t += 1
    rest = [(i, j) for i, n in enumerate(sizes) for j in range(t, n)]
    if rest:
        out.append(rest)
    return out


def multicast_steps(b, n_nodes):
    """Steps of a 1 -> n_nodes binomial-pipeline multicast of b blocks."""
    log = 0
    while (1 << log) < n_nodes:
        log += 1
    return b + log - 1


def multicast_schedule(b, n_nodes):
    """1 -> n_nodes multicast of b blocks from node 0, n_nodes a power of two.  Returns a list
    of steps; step s is a dict {sender: (receiver, block)}.  In step s every node u is paired
    with u XOR 2^(s mod n); node 0 offers block s while there are new ones, every other node
    (and node 0 afterwards) the highest-numbered block it holds that its partner lacks.  All
    transfers of a step happen at once."""
    n = n_nodes.bit_length() - 1
    assert n_nodes == 1 << n and b >= 1
    have = [set() for _ in range(n_nodes)]
    have[0] = set(range(b))
    steps = []
    while any(len(h) < b for h in have):
        s = len(steps)
        bit = 1 << (s % n)
        sends = {}
        for u in range(n_nodes):
            v = u ^ bit
            useful = [k for k in have[u] if k not in have[v]]
            if not useful:
                continue
            k = max(useful)
            if u == 0 and min(s, b - 1) in useful:
                k = min(s, b - 1)
            sends[u] = (v, k)
        for u, (v, k) in sends.items():
            have[v].add(k)
        steps.append(sends)
    return steps
