"""Oracle for the cluster-level KV placement step: performance model and greedy scheduler.

TEST INFRASTRUCTURE ONLY.  Plain Python floats (fp64), written from Section 5.2 / 5.3 (Eq. 5, 6, 7 and the greedy
rule of Algorithm 1, stated here as a definition: roles, the request that gives blocks, the admissible block counts,
the argmax, the order of offers) in the paper's notation; nothing here is shared with the C++ implementation.

Notation: beta = batch size of an instance, S^r = length of request r in tokens, g = attention rate in tokens per
second (a constant, Section 5.3), T^natn(beta) = W(beta) / f(beta) = measured time of the non-attention part of one
layer at batch size beta (given as a table), n = number of layers, K^d / K^c = tokens of KV cache a debtor has placed
on creditors / a creditor holds for debtors.

Readings where the paper is silent (each is also listed in the design notes):
  * beta' of Eq. 6: memory that a debtor frees lets it admit queued requests.  An instance states how many requests
    wait (`waiting`) and how many blocks one of them needs (`admit_blocks`); it admits as many as fit in its free
    blocks, each adding admit_blocks * block_tokens tokens to its attention work.
  * Section 5.2 forbids an instance to be debtor and creditor at once: an instance with utilisation <= U^thres is a
    creditor; a debtor is an instance with beta <= beta^thres that is not a creditor, holds at least one request
    and hosts nothing; an instance that has lent blocks out is no creditor.
  * k ranges over 0 .. Block_max - 1 as the listing's range(0, Block_max) says, so the request's last block (where
    new tokens are appended) stays with the debtor; k is also bounded by the creditor's free blocks.
  * pick_max_perf takes the smallest k among equal maxima, so "no gain" gives 0 and ends the debtor's loop.
  * after a move the creditors not yet tried by this debtor are re-sorted by utilisation; each creditor is tried
    at most once per debtor; ties in any sort go to the lower instance index.
  * one request (the longest) per debtor per invocation, as listed.
"""


class Instance:
    """Mutable state of one serving instance."""

    def __init__(self, req_tokens, capacity_blocks, req_remote_blocks=None, hosted_blocks=0, waiting=0, admit_blocks=0):
        self.req_tokens = list(req_tokens)
        self.req_remote_blocks = list(req_remote_blocks) if req_remote_blocks is not None else [0] * len(self.req_tokens)
        self.hosted_blocks = hosted_blocks
        self.capacity_blocks = capacity_blocks
        self.waiting = waiting
        self.admit_blocks = admit_blocks
        self.admitted = 0  # requests admitted from the queue during scheduling

    def copy(self):
        c = Instance(self.req_tokens, self.capacity_blocks, self.req_remote_blocks, self.hosted_blocks, self.waiting,
                     self.admit_blocks)
        c.admitted = self.admitted
        return c


class Model:
    def __init__(self, num_layers, block_tokens, attn_tokens_per_s, t_natn):
        self.n = num_layers
        self.T = block_tokens
        self.g = attn_tokens_per_s
        self.t_natn = list(t_natn)  # t_natn[b] = seconds per layer of non-attention work at batch size b


def blocks_of(model, tokens):
    return -(-tokens // model.T)


def batch(inst):
    """beta: own requests plus the ones admitted from the queue."""
    return len(inst.req_tokens) + inst.admitted


def own_tokens(model, inst):
    """Sum over the instance's requests of S^r (admitted requests count admit_blocks full blocks each)."""
    return sum(inst.req_tokens) + inst.admitted * inst.admit_blocks * model.T


def remote_blocks(inst):
    return sum(inst.req_remote_blocks)


def remote_tokens(model, inst):
    """K^d in tokens: remote blocks are full except a request's last block, which goes last."""
    return sum(min(rb * model.T, s) for s, rb in zip(inst.req_tokens, inst.req_remote_blocks))


def used_blocks(model, inst):
    own = sum(blocks_of(model, s) for s in inst.req_tokens) + inst.admitted * inst.admit_blocks
    return own - remote_blocks(inst) + inst.hosted_blocks


def utilisation(model, inst):
    return used_blocks(model, inst) / inst.capacity_blocks


def layer_time(model, beta, attn_tokens):
    """Eq. 5: T^lyr(beta, S) = T^natn(beta) + sum_r S^r / g."""
    return model.t_natn[beta] + attn_tokens / model.g


def admit_count(model, inst, k):
    """Requests a debtor can admit from its queue once k more blocks have left (reading of beta' in Eq. 6)."""
    if inst.admit_blocks <= 0 or inst.waiting <= 0:
        return 0
    free = inst.capacity_blocks - used_blocks(model, inst) + k
    a = min(inst.waiting, free // inst.admit_blocks) if free > 0 else 0
    room = len(model.t_natn) - 1 - batch(inst)
    return max(0, min(a, room))


def debtor_tps(model, inst, k):
    """Eq. 6 (debtor) and TPS = beta' / (n T): the debtor with k more blocks placed remotely."""
    a = admit_count(model, inst, k)
    beta2 = batch(inst) + a
    if beta2 == 0:
        return 0.0
    tokens = own_tokens(model, inst) + a * inst.admit_blocks * model.T
    k_d = remote_tokens(model, inst) + k * model.T
    k_c = inst.hosted_blocks * model.T  # zero for an instance in the debtor role; kept so that k = 0 is the present state
    t = layer_time(model, beta2, tokens) - k_d / model.g + k_c / model.g
    return beta2 / (model.n * t)


def creditor_tps(model, inst, k):
    """Eq. 6 (creditor) and TPS = beta / (n T): the creditor hosting k more blocks."""
    beta = batch(inst)
    if beta == 0:
        return 0.0
    k_own_remote = remote_tokens(model, inst)
    k_c = (inst.hosted_blocks + k) * model.T
    t = layer_time(model, beta, own_tokens(model, inst)) - k_own_remote / model.g + k_c / model.g
    return beta / (model.n * t)


def instance_tps(model, inst):
    """Throughput of an instance in its current state: TPS = beta / (n T) with both adjustments of Eq. 6."""
    beta = batch(inst)
    if beta == 0:
        return 0.0
    t = layer_time(model, beta, own_tokens(model, inst)) - remote_tokens(model, inst) / model.g \
        + inst.hosted_blocks * model.T / model.g
    return beta / (model.n * t)


def cluster_tps(model, instances):
    """Eq. 7."""
    return sum(instance_tps(model, i) for i in instances)


def pair_estimate(model, debtor, creditor, k):
    """perf_model_throughput_esti(k, D, C) of Algorithm 1: aggregated throughput of the two instances (Eq. 7)."""
    return debtor_tps(model, debtor, k) + creditor_tps(model, creditor, k)


def apply_move(model, debtor, r, creditor, k):
    """move_kvcache: k blocks of request r go from the debtor to the creditor; the debtor admits what now fits."""
    a = admit_count(model, debtor, k)
    debtor.req_remote_blocks[r] += k
    debtor.admitted += a
    debtor.waiting -= a
    creditor.hosted_blocks += k


def is_creditor(model, inst, u_thres):
    """Section 5.2: spare memory (utilisation at most U^thres) and nothing of its own placed elsewhere."""
    return utilisation(model, inst) <= u_thres and remote_blocks(inst) == 0


def is_debtor(model, inst, beta_thres, u_thres):
    """Section 5.2: a small batch (at most beta^thres) on an instance that is no creditor, has a request to give
    blocks from and hosts nothing for others."""
    return (batch(inst) <= beta_thres and not is_creditor(model, inst, u_thres) and len(inst.req_tokens) > 0
            and inst.hosted_blocks == 0)


def longest_request(inst):
    """The request a debtor gives blocks from; the lower index among equally long ones."""
    return min(range(len(inst.req_tokens)), key=lambda r: (-inst.req_tokens[r], r))


def movable_blocks(model, debtor, r, creditor):
    """The block counts k the rule may choose from: 0 up to what the creditor has free, and never the request's
    last local block (new tokens are appended there)."""
    local = blocks_of(model, debtor.req_tokens[r]) - debtor.req_remote_blocks[r]
    free = creditor.capacity_blocks - used_blocks(model, creditor)
    return range(0, max(0, min(local, free + 1)))


def blocks_to_move(model, debtor, r, creditor):
    """The greedy choice: the k whose estimate for the pair (Eq. 6 for both, summed as in Eq. 7) is largest; the
    smallest such k, so that "nothing gained" is 0."""
    ks = movable_blocks(model, debtor, r, creditor)
    return max(ks, key=lambda k: (pair_estimate(model, debtor, creditor, k), -k)) if len(ks) else 0


def schedule(model, instances, beta_thres, u_thres):
    """The placement rule of Section 5.3 stated as a definition.  Returns (moves, instances_after); a move is
    (debtor, request, creditor, blocks).

    Debtors are served in order of batch size.  A debtor offers blocks of its longest request to the creditors one
    at a time, always to the least utilised creditor it has not offered to yet (utilisations as they stand then);
    the number of blocks that creditor takes is blocks_to_move; the first creditor that takes none ends the
    debtor's turn."""
    inst = [i.copy() for i in instances]
    everyone = range(len(inst))
    creditors = [c for c in everyone if is_creditor(model, inst[c], u_thres)]
    debtors = sorted((d for d in everyone if is_debtor(model, inst[d], beta_thres, u_thres)), key=lambda d: (batch(inst[d]), d))
    moves = []

    def offer(d, r, asked):
        open_to = [c for c in creditors if c not in asked]
        if not open_to:
            return
        c = min(open_to, key=lambda x: (utilisation(model, inst[x]), x))
        k = blocks_to_move(model, inst[d], r, inst[c])
        if k == 0:
            return
        apply_move(model, inst[d], r, inst[c], k)
        moves.append((d, r, c, k))
        offer(d, r, asked | {c})

    for d in debtors:
        offer(d, longest_request(inst[d]), frozenset())
    return moves, inst
