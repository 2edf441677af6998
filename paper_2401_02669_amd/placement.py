"""ctypes binding of the cluster-level placement entry points (include/distattn_placement.h).  Marshalling only."""
import ctypes

from . import distattn as da

EXPORTS = ["da_model_instance_tps", "da_model_cluster_tps", "da_model_pair_estimate", "da_placement_schedule"]


class DaPerfModel(ctypes.Structure):
    _fields_ = [("num_layers", ctypes.c_int32), ("block_tokens", ctypes.c_int32), ("attn_tokens_per_s", ctypes.c_double),
                ("t_natn", ctypes.POINTER(ctypes.c_double)), ("t_natn_len", ctypes.c_int32)]


class DaInstance(ctypes.Structure):
    _fields_ = [("num_requests", ctypes.c_int32), ("req_tokens", ctypes.POINTER(ctypes.c_int64)),
                ("req_remote_blocks", ctypes.POINTER(ctypes.c_int32)), ("hosted_blocks", ctypes.c_int32),
                ("capacity_blocks", ctypes.c_int32), ("waiting", ctypes.c_int32), ("admit_blocks", ctypes.c_int32)]


class DaMove(ctypes.Structure):
    _fields_ = [("debtor", ctypes.c_int32), ("request", ctypes.c_int32), ("creditor", ctypes.c_int32),
                ("blocks", ctypes.c_int32)]


_ready = False


def _lib():
    global _ready
    L = da.lib()
    if not _ready:
        dp = ctypes.POINTER(ctypes.c_double)
        mp, ip = ctypes.POINTER(DaPerfModel), ctypes.POINTER(DaInstance)
        L.da_model_instance_tps.argtypes = [mp, ip, dp]
        L.da_model_cluster_tps.argtypes = [mp, ip, ctypes.c_int32, dp]
        L.da_model_pair_estimate.argtypes = [mp, ip, ip, ctypes.c_int32, dp]
        L.da_placement_schedule.argtypes = [mp, ip, ctypes.c_int32, ctypes.c_int32, ctypes.c_double,
                                            ctypes.POINTER(DaMove), ctypes.c_int32, ctypes.POINTER(ctypes.c_int32), dp, dp]
        for name in EXPORTS:
            getattr(L, name).restype = ctypes.c_int
        _ready = True
    return L


class Model:
    """Holds a da_perf_model and the table it points to."""

    def __init__(self, num_layers, block_tokens, attn_tokens_per_s, t_natn):
        self._table = (ctypes.c_double * len(t_natn))(*t_natn)
        self.c = DaPerfModel(num_layers, block_tokens, attn_tokens_per_s,
                             ctypes.cast(self._table, ctypes.POINTER(ctypes.c_double)), len(t_natn))


class Cluster:
    """Holds an array of da_instance and the arrays they point to."""

    def __init__(self, instances):
        n = len(instances)
        self.c = (DaInstance * n)()
        self._keep = []
        for i, d in enumerate(instances):
            toks = (ctypes.c_int64 * max(1, len(d["req_tokens"])))(*d["req_tokens"])
            rem = d.get("req_remote_blocks")
            self._keep.append(toks)
            self.c[i].num_requests = len(d["req_tokens"])
            self.c[i].req_tokens = ctypes.cast(toks, ctypes.POINTER(ctypes.c_int64))
            if rem is not None:
                rem_c = (ctypes.c_int32 * max(1, len(rem)))(*rem)
                self._keep.append(rem_c)
                self.c[i].req_remote_blocks = ctypes.cast(rem_c, ctypes.POINTER(ctypes.c_int32))
            self.c[i].hosted_blocks = d.get("hosted_blocks", 0)
            self.c[i].capacity_blocks = d["capacity_blocks"]
            self.c[i].waiting = d.get("waiting", 0)
            self.c[i].admit_blocks = d.get("admit_blocks", 0)

    def __len__(self):
        return len(self.c)


def instance_tps(model, cluster, i):
    v = ctypes.c_double()
    da._check(_lib().da_model_instance_tps(ctypes.byref(model.c), ctypes.byref(cluster.c[i]), ctypes.byref(v)),
              "da_model_instance_tps")
    return v.value


def cluster_tps(model, cluster):
    v = ctypes.c_double()
    da._check(_lib().da_model_cluster_tps(ctypes.byref(model.c), cluster.c, len(cluster), ctypes.byref(v)),
              "da_model_cluster_tps")
    return v.value


def pair_estimate(model, cluster, debtor, creditor, k):
    v = ctypes.c_double()
    da._check(_lib().da_model_pair_estimate(ctypes.byref(model.c), ctypes.byref(cluster.c[debtor]),
                                            ctypes.byref(cluster.c[creditor]), k, ctypes.byref(v)), "da_model_pair_estimate")
    return v.value


def schedule(model, cluster, beta_thres, u_thres, max_moves=None):
    """Algorithm 1: returns (moves, tps_before, tps_after); a move is (debtor, request, creditor, blocks)."""
    if max_moves is None:
        max_moves = len(cluster) * len(cluster)
    moves = (DaMove * max(1, max_moves))()
    n = ctypes.c_int32()
    before, after = ctypes.c_double(), ctypes.c_double()
    da._check(_lib().da_placement_schedule(ctypes.byref(model.c), cluster.c, len(cluster), beta_thres, u_thres, moves,
                                           max_moves, ctypes.byref(n), ctypes.byref(before), ctypes.byref(after)),
              "da_placement_schedule")
    return [(m.debtor, m.request, m.creditor, m.blocks) for m in moves[:n.value]], before.value, after.value
