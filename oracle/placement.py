"""Oracle for the cluster-level KV placement step: performance model and greedy scheduler.

TEST INFRASTRUCTURE ONLY.  Plain Python floats (fp64) and loops, written from Section 5.3 (Eq. 5, 6, 7 and
Algorithm 1) in the paper's order and notation; nothing here is shared with the C++ implementation.

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


def schedule(model, instances, beta_thres, u_thres):
    """Algorithm 1.  Returns (moves, instances_after); a move is (debtor, request, creditor, blocks)."""
    inst = [i.copy() for i in instances]
    M = len(inst)
    is_creditor = [utilisation(model, inst[i]) <= u_thres and remote_blocks(inst[i]) == 0 for i in range(M)]
    debtors = [i for i in range(M)
               if batch(inst[i]) <= beta_thres and not is_creditor[i] and len(inst[i].req_tokens) > 0
               and inst[i].hosted_blocks == 0]
    debtors.sort(key=lambda i: (batch(inst[i]), i))
    creditors = [i for i in range(M) if is_creditor[i]]
    moves = []
    for d in debtors:
        D = inst[d]
        r = max(range(len(D.req_tokens)), key=lambda x: (D.req_tokens[x], -x))
        block_max = blocks_of(model, D.req_tokens[r]) - D.req_remote_blocks[r]
        tried = set()
        while True:
            order = sorted((c for c in creditors if c not in tried), key=lambda c: (utilisation(model, inst[c]), c))
            if not order:
                break
            c = order[0]
            tried.add(c)
            C = inst[c]
            free_c = C.capacity_blocks - used_blocks(model, C)
            best_k, best_perf = 0, None
            for k in range(0, block_max):
                if k > free_c:
                    break
                perf = pair_estimate(model, D, C, k)
                if best_perf is None or perf > best_perf:
                    best_k, best_perf = k, perf
            if best_k <= 0:
                break
            apply_move(model, D, r, C, best_k)
            moves.append((d, r, c, best_k))
            block_max -= best_k
    return moves, inst
