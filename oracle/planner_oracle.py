"""CPU oracle of the paper's planning steps (test infrastructure only: tests import it, the
product never does).  Plain Python, integers only.

  * k-way transmission order: Section 4.2, Algorithm 1.
  * sub-group sizes for k -> N scaling: Section 4.2, "Multicast and sub-groups".
  * execution pipeline generation: Section 4.3, Algorithm 2.
  * number of multicast steps of the binomial pipeline: Section 4.2 (b + ceil(log2 N) - 1).

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
    the order they are formed, each a list of (sub-group, node index inside it)."""
    used = [0] * len(sizes)
    out = []
    while True:
        live = [i for i in range(len(sizes)) if used[i] < sizes[i]]
        if not live:
            return out
        if len(live) == 1:
            g = live[0]
            out.append([(g, j) for j in range(used[g], sizes[g])])
            used[g] = sizes[g]
            continue
        a = min(sizes[i] - used[i] for i in live)
        for _ in range(a):
            out.append([(i, used[i]) for i in live])
            for i in live:
                used[i] += 1


def multicast_steps(b, n_nodes):
    """Steps of a 1 -> n_nodes binomial-pipeline multicast of b blocks."""
    log = 0
    while (1 << log) < n_nodes:
        log += 1
    return b + log - 1
