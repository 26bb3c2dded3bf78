"""CPU oracle of the cache manager and the cache swapper (paper sections 4 and 5).

TEST INFRASTRUCTURE ONLY: a plain, slow, obviously correct model of the host logic that
produces the block lists of the hot path.  Only tests/, the smoke test and bench.py's
cpu_baseline leg may import it; the product path (libflpool.so) shares no code with it.

What it models, in the paper's order:

* Section 4.1: one tree; a virtual root, the LoRA nodes on the second layer (label: LoRA id),
  below each LoRA the KV caches of the conversations that used it (label: token sequence).
  Here a KV node is one pool block, i.e. `block_tokens` consecutive tokens; only full blocks
  become nodes.
* Section 4.2: a query first matches its LoRA node, then walks down the KV nodes that spell its
  tokens until a leaf or a miss; what is matched on the host tier is swapped in (top down);
  what the query computes anew is inserted below the last matched node and stays in HBM.
  Swap-out starts from the leaves that are in HBM, swap-in from the roots of the sub-trees
  that are in host memory, so an HBM-resident node never has a non-resident ancestor.
* Section 4.3: every node keeps visit frequency, time of last use and size.
* Section 5.1, Eq. 3: Low_lora = sum_i 1 - (1 - prob_i)^BS.
* Section 5.2, Eq. 4: LoRA_Eval = max(1, Low_lora / Now_LoRA);
  Eq. 5: Retain_Eval_i = cost_i * prob_i * (1 - sigmoid(t_i)); Eq. 6: Eval_i = LoRA_Eval_i * Retain_Eval_i.
* Section 5.3: every monitor interval the HBM usage is compared with an upper and a lower
  threshold; above the upper one the candidates (HBM leaves) are swapped out in increasing order
  of Eval, below the lower one the candidates (host roots) are swapped in in decreasing order,
  one by one, until the usage is back between the thresholds.
* Sections 6.6-6.8 (ablations): LRU instead of the cost model, no dependencies (every node is
  a candidate), no LoRA reward.

Readings where the paper is silent are listed in the design notes; the ones that matter here:
prob_i = visits_i / number of matched queries; LoRA_Eval applies to LoRA nodes only (1 for KV
nodes) with Now_LoRA taken as at least 1; Low_lora and Now_LoRA are sampled once per tick;
t_i = (now - last use) / time_scale; ties in Eval go to the older node (lower id); nodes in
use by a running query are not candidates; "balanced" = usage <= upper after swap-out,
usage >= lower after swap-in (never exceeding upper).
"""
import math

HBM, HOST = 0, 1
LORA, KV = 0, 1


class Lifo:
    """The pool's free list of one tier (paper section 4.3: freed blocks are recycled): the first n
    allocations return 0, 1, 2, ...; the block freed last is handed out first."""

    def __init__(self, n):
        self.n = n
        self.stack = list(range(n - 1, -1, -1))
        self.is_free = [True] * n

    def num_free(self):
        return len(self.stack)

    def alloc(self, n):
        if n > len(self.stack):
            return None
        out = [self.stack.pop() for _ in range(n)]
        for i in out:
            self.is_free[i] = False
        return out

    def free(self, ids):
        for i in ids:
            assert 0 <= i < self.n and not self.is_free[i]
            self.is_free[i] = True
            self.stack.append(i)


class Node:
    def __init__(self, nid, kind, key, parent, tier, blocks, now):
        self.id, self.kind, self.key, self.parent = nid, kind, key, parent
        self.tier, self.blocks = tier, list(blocks)
        self.children = {}
        self.visits, self.last_use, self.pins = 0, now, 0


class CacheOracle:
    def __init__(self, n_dev_blocks, n_host_blocks, block_tokens=16, block_bytes=262144, upper=0.95, lower=0.70,
                 pcie_bytes_per_s=64e9, time_scale_s=60.0, use_lru=False, ignore_dependencies=False,
                 no_lora_reward=False):
        self.free = [Lifo(n_dev_blocks), Lifo(n_host_blocks)]
        self.n_dev = n_dev_blocks
        self.bt, self.block_bytes = block_tokens, block_bytes
        self.upper, self.lower = upper, lower
        self.bw, self.tau = pcie_bytes_per_s, time_scale_s
        self.use_lru, self.no_dep, self.no_reward = use_lru, ignore_dependencies, no_lora_reward
        self.root = Node(0, LORA, None, None, HBM, [], 0.0)
        self.nodes = {0: self.root}
        self.next_id = 1
        self.n_queries = 0
        self.queries = {}
        self.next_query = 1

    # ------------------------------------------------------------------ tree (sections 4.1-4.3)
    def usage(self):
        return 1.0 - self.free[HBM].num_free() / self.n_dev

    def _new_node(self, kind, key, parent, tier, blocks, now):
        n = Node(self.next_id, kind, key, parent, tier, blocks, now)
        self.nodes[n.id] = n
        self.next_id += 1
        parent.children[key] = n
        return n

    def add_lora(self, lora_id, n_blocks, tier, now):
        """A LoRA enters the pool on `tier` (its pages split along the rank dimension over n_blocks
        blocks).  Returns its block ids, or None when the tier has too few free blocks."""
        assert lora_id not in self.root.children
        ids = self.free[tier].alloc(n_blocks)
        if ids is None:
            return None
        self._new_node(LORA, lora_id, self.root, tier, ids, now)
        return ids

    def match(self, lora_id, tokens, now):
        """Section 4.2: match the LoRA node, then the KV nodes spelling `tokens`, top down.  Matched
        nodes on the host tier are swapped in as far as HBM has room (a node is usable only with all
        its ancestors resident, so the match ends at the first node that cannot be brought in).
        Returns (query handle, lora block ids or None, matched KV block ids, swap_in pairs).
        lora block ids is None when the LoRA itself could not be brought into HBM (the query waits)."""
        lora = self.root.children[lora_id]
        path = [lora]
        node = lora
        for b in range(len(tokens) // self.bt):
            key = tuple(tokens[b * self.bt:(b + 1) * self.bt])
            child = node.children.get(key)
            if child is None:
                break
            path.append(child)
            node = child
        self.n_queries += 1
        swap_in, usable = [], []
        for n in path:
            n.visits += 1
            n.last_use = now
        for n in path:
            if n.tier == HOST:
                ids = self.free[HBM].alloc(len(n.blocks))
                if ids is None:
                    break
                swap_in += list(zip(n.blocks, ids))
                self.free[HOST].free(n.blocks)
                n.tier, n.blocks = HBM, ids
            usable.append(n)
        for n in usable:
            n.pins += 1
        q = self.next_query
        self.next_query += 1
        self.queries[q] = usable
        lora_blocks = list(lora.blocks) if usable else None
        kv_blocks = [n.blocks[0] for n in usable[1:]]
        return q, lora_blocks, kv_blocks, swap_in

    def insert(self, query, tokens, new_blocks, now):
        """Section 4.2: the KV blocks the query filled (full blocks of its tokens past the matched
        prefix, already in HBM, ids in `new_blocks`) become nodes below the last matched node and are
        pinned by the query like the matched ones.  Returns the ids that were NOT taken over because a
        node with the same tokens already exists (the caller frees them)."""
        path = self.queries[query]
        if not path:
            return list(new_blocks)
        node = path[-1]
        first = len(path) - 1                      # KV blocks the query holds so far
        not_taken = []
        for j, blk in enumerate(new_blocks):
            b = first + j
            key = tuple(tokens[b * self.bt:(b + 1) * self.bt])
            assert len(key) == self.bt
            child = node.children.get(key)
            if child is None:
                child = self._new_node(KV, key, node, HBM, [blk], now)
                child.visits = 1
            elif child.tier == HBM:
                not_taken.append(blk)              # somebody else inserted the same continuation first
                child.visits += 1
                child.last_use = now
            else:
                # the same continuation exists on the host tier: a resident chain cannot go on below it
                return not_taken + list(new_blocks[j:])
            child.pins += 1
            path.append(child)
            node = child
        return not_taken

    def release(self, query):
        for n in self.queries.pop(query):
            n.pins -= 1

    # ------------------------------------------------------------------ cost model (section 5)
    def lora_nodes(self):
        return sorted(self.root.children.values(), key=lambda n: n.id)

    def prob(self, n):
        return n.visits / self.n_queries if self.n_queries else 0.0

    def low_lora(self, batch_size):
        """Eq. 3."""
        return sum(1.0 - (1.0 - self.prob(n)) ** batch_size for n in self.lora_nodes())

    def now_lora(self):
        return sum(1 for n in self.lora_nodes() if n.tier == HBM)

    def lora_eval(self, low, now_lora):
        """Eq. 4."""
        return max(1.0, low / max(now_lora, 1))

    def retain_eval(self, n, now):
        """Eq. 5."""
        cost = len(n.blocks) * self.block_bytes / self.bw
        t = (now - n.last_use) / self.tau
        return cost * self.prob(n) * (1.0 - 1.0 / (1.0 + math.exp(-t)))

    def eval(self, n, now, low, now_lora):
        """Eq. 6 (or the last use time under the LRU ablation)."""
        if self.use_lru:
            return n.last_use
        reward = self.lora_eval(low, now_lora) if (n.kind == LORA and not self.no_reward) else 1.0
        return reward * self.retain_eval(n, now)

    # ------------------------------------------------------------------ swapper (section 5.3)
    def _real_nodes(self):
        return [n for n in self.nodes.values() if n is not self.root]

    def out_candidates(self):
        """HBM nodes that no running query uses and that have no child in HBM (section 4.2: swap-out
        starts from the leaves in HBM); every unused HBM node when dependencies are ignored."""
        out = []
        for n in self._real_nodes():
            if n.tier != HBM or n.pins:
                continue
            if self.no_dep or not any(c.tier == HBM for c in n.children.values()):
                out.append(n)
        return out

    def in_candidates(self):
        """Host nodes whose parent is in HBM (section 4.2: swap-in starts from the roots of the
        sub-trees in main memory); every host node when dependencies are ignored."""
        return [n for n in self._real_nodes()
                if n.tier == HOST and (self.no_dep or n.parent is self.root or n.parent.tier == HBM)]

    def tick(self, now, batch_size):
        """One monitor interval.  Returns (swap_out pairs (dev id, host id), swap_in pairs (host id,
        dev id), dropped node ids) in the order the moves are decided."""
        low, now_lora = self.low_lora(batch_size), self.now_lora()
        key = lambda n: (self.eval(n, now, low, now_lora), n.id)
        swap_out, swap_in, dropped = [], [], []
        if self.usage() > self.upper:
            while self.usage() > self.upper:
                cand = self.out_candidates()
                if not cand:
                    break
                n = min(cand, key=key)
                ids = self.free[HOST].alloc(len(n.blocks))
                self.free[HBM].free(n.blocks)
                if ids is None:
                    # no room on the host tier: a node without children is forgotten, any other stays put
                    # on paper but its blocks are gone, so its whole sub-tree is forgotten with it
                    dropped += self._drop(n)
                    continue
                swap_out += list(zip(n.blocks, ids))
                n.tier, n.blocks = HOST, ids
        elif self.usage() < self.lower:
            while self.usage() < self.lower:
                cand = self.in_candidates()
                if not cand:
                    break
                n = min(cand, key=lambda m: (-key(m)[0], m.id))
                if 1.0 - (self.free[HBM].num_free() - len(n.blocks)) / self.n_dev > self.upper:
                    break
                ids = self.free[HBM].alloc(len(n.blocks))
                if ids is None:
                    break
                swap_in += list(zip(n.blocks, ids))
                self.free[HOST].free(n.blocks)
                n.tier, n.blocks = HBM, ids
        return swap_out, swap_in, dropped

    def _drop(self, n):
        """Forget n and everything below it (their blocks return to the free lists; n's own HBM
        blocks were already returned by the caller)."""
        gone = []
        stack = [n]
        first = True
        while stack:
            m = stack.pop()
            stack += sorted(m.children.values(), key=lambda c: -c.id)
            if not first:
                self.free[m.tier].free(m.blocks)
            first = False
            gone.append(m.id)
            del self.nodes[m.id]
        del n.parent.children[n.key]
        return gone

    # ------------------------------------------------------------------ statistics
    def invalid_kv_blocks(self):
        """HBM-resident KV blocks that cannot be matched because an ancestor is not in HBM."""
        bad = 0
        for n in self._real_nodes():
            if n.kind == KV and n.tier == HBM:
                p = n.parent
                while p is not self.root and p.tier == HBM:
                    p = p.parent
                if p is not self.root:
                    bad += len(n.blocks)
        return bad

    def snapshot(self):
        """Everything observable, for comparisons: per node (id, kind, parent id, tier, blocks, visits,
        last use, pins), sorted by id."""
        return [(n.id, n.kind, n.parent.id, n.tier, tuple(n.blocks), n.visits, n.last_use, n.pins)
                for n in sorted(self._real_nodes(), key=lambda n: n.id)]
