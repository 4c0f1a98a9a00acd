"""The oracle's own reader for `monet-graph` and `monet-schedule` text (test infrastructure).

Nodes 1..N are the forward operators of Section 3 in topological order with
their incoming edges N_j; backward operators k = 1..B each belong to one
forward node and list, per implementation, workspace, cost and the forward
tensors D_k^l they read (Section 4, "Backward Operator Optimization").
"""
from dataclasses import dataclass, field

ALIGN = 256          # logical size of a tensor = bytes rounded up to this


def align(b):
    return (int(b) + ALIGN - 1) // ALIGN * ALIGN


def _dims(s):
    return tuple(int(d) for d in s.split("x"))


def _refs(s):
    return [] if s == "-" else [int(v) for v in s.split(",")]


def _kv(fields):
    out = {}
    for f in fields:
        k, v = f.split("=", 1)
        out[k] = v
    return out


@dataclass
class ONode:
    id: int
    op: str
    ins: list
    pars: list
    shape: tuple
    attrs: dict
    fimpls: list = field(default_factory=list)   # [dict(algo, ws, cost, inplace)]

    @property
    def is_aux(self):
        return self.op in ("mask", "poolidx")

    @property
    def persist(self):
        return self.attrs.get("persist") == "1"


@dataclass
class OBop:
    k: int
    kind: str
    node: int
    impls: list = field(default_factory=list)    # [dict(algo, deps, ws, cost)]


class OGraph:
    def __init__(self, text):
        self.exts = {}      # ref -> (name, dtype, shape)
        self.params = {}    # pid -> (name, shape)
        self.nodes = {}     # i -> ONode
        self.bops = {}      # k -> OBop
        lines = [ln.split("#")[0].split() for ln in text.splitlines()]
        lines = [ln for ln in lines if ln]
        if lines[0] != ["monet-graph", "1"]:
            raise ValueError("not a monet-graph 1 text")
        for f in lines[1:]:
            tag = f[0]
            if tag == "ext":
                self.exts[int(f[1])] = (f[2], f[3], _dims(f[4]))
            elif tag == "param":
                self.params[int(f[1])] = (f[2], _dims(f[3]))
            elif tag == "node":
                kv = _kv(f[3:])
                n = ONode(int(f[1]), f[2], _refs(kv.pop("in")), _refs(kv.pop("par")), _dims(kv.pop("shape")), kv)
                self.nodes[n.id] = n
            elif tag == "fimpl":
                kv = _kv(f[3:])
                n = self.nodes[int(f[1])]
                assert int(f[2]) == len(n.fimpls)
                n.fimpls.append(dict(algo=kv["algo"], ws=int(kv["ws"]), cost=float(kv["cost"]),
                                     inplace=kv.get("inplace") == "1", extra=kv))
            elif tag == "bop":
                kv = _kv(f[3:])
                self.bops[int(f[1])] = OBop(int(f[1]), f[2], int(kv["node"]))
            elif tag == "bimpl":
                kv = _kv(f[3:])
                b = self.bops[int(f[1])]
                assert int(f[2]) == len(b.impls)
                b.impls.append(dict(algo=kv["algo"], deps=_refs(kv["deps"]), ws=int(kv["ws"]),
                                    cost=float(kv["cost"]), extra=kv))
            else:
                raise ValueError(f"unknown record {tag}")
        self.N = len(self.nodes)
        self.B = len(self.bops)
        assert sorted(self.nodes) == list(range(1, self.N + 1))
        assert sorted(self.bops) == list(range(1, self.B + 1))
        for n in self.nodes.values():
            for j in n.ins:
                assert j < n.id, "edges must point forward"
        # consumers among real (non-aux) operators
        self.consumers = {i: [] for i in self.nodes}
        for n in self.nodes.values():
            if not n.is_aux:
                for j in n.ins:
                    if j > 0:
                        self.consumers[j].append(n.id)
        self.aux_children = {i: [] for i in self.nodes}
        for n in self.nodes.values():
            if n.is_aux:
                self.aux_children[n.ins[0]].append(n.id)

    def nbytes(self, i):
        """|x_i|: logical bytes of node i's output."""
        n = self.nodes[i]
        if n.persist:
            return 0
        cnt = 1
        for d in n.shape:
            cnt *= d
        size = {"mask": 8, "poolidx": 1}.get(n.op, 4)
        return align(cnt * size)

    def shape_of(self, ref):
        return self.exts[ref][2] if ref <= 0 else self.nodes[ref].shape


class OSchedule:
    def __init__(self, text, g: OGraph):
        self.fwd_impl = {}
        self.fwd_save = set()
        self.stage_impl = {}
        self.r = {k: {} for k in range(1, g.B + 1)}
        self.s = {k: set() for k in range(1, g.B + 1)}
        lines = [ln.split("#")[0].split() for ln in text.splitlines()]
        lines = [ln for ln in lines if ln]
        if lines[0] != ["monet-schedule", "1"]:
            raise ValueError("not a monet-schedule 1 text")
        for f in lines[1:]:
            if f[0] == "fwd":
                kv = _kv(f[2:])
                self.fwd_impl[int(f[1])] = int(kv["impl"])
                if kv["save"] == "1":
                    self.fwd_save.add(int(f[1]))
            elif f[0] == "stage":
                self.stage_impl[int(f[1])] = int(_kv(f[2:])["impl"])
            elif f[0] == "r":
                self.r[int(f[1])][int(f[2])] = int(_kv(f[3:])["impl"])
            elif f[0] == "s":
                self.s[int(f[1])].add(int(f[2]))
            else:
                raise ValueError(f"unknown record {f[0]}")
        assert sorted(self.fwd_impl) == list(range(1, g.N + 1))
        assert sorted(self.stage_impl) == list(range(1, g.B + 1))

    def saved_entering(self, k, B):
        """S^k: what stage k starts from (the forward pass's S^N for the first stage)."""
        return self.fwd_save if k == B else self.s[k + 1]
