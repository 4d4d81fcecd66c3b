"""CPU oracle for the train<->generation weight reshard of the 3D-HybridEngine.

THIS IS TEST INFRASTRUCTURE.  Only tests/, __graft_entry__.smoke() and the
`cpu_baseline` leg of bench.py may import it.  It shares no code with the HIP
library (paper_2409_19256_amd/): it computes every offset, group and index itself.

What is computed, and from which passage of the HybridFlow paper (arXiv 2409.19256):

* Training parallel groups p-t-d: TP and PP groups are consecutive ranks, DP groups
  are ranks at stride p*t (Section 5.3, first paragraph; Figure 8(a)).
* Generation parallel groups p_g-t_g-d_g-d with d_g = p*t/(p_g*t_g) (Section 5.1).
  "hybridflow" grouping: generation TP / PP groups take ranks at stride t/t_g and
  p/p_g, micro-DP groups are consecutive ranks (Section 5.3, Figure 8(b)).
  "vanilla" grouping (HybridFlow-V): the training rule with the smaller sizes
  (Section 5.3, Figure 8(a)).
* Step 1 of the workflow (Section 5.2, Figure 7): every rank obtains its generation
  partition from the training shards of its micro-DP group.  Because the result is
  a pure re-arrangement of bytes it has a plain definition, which is what is
  written here: rebuild each FULL logical tensor from ALL training shards by
  concatenation along the Megatron column-/row-parallel axis, then slice out what
  the generation rank holds.  No attempt is made to touch only the needed shards.
* Step 4 (Section 5.2): re-partition for training = rebuild the full tensors from
  the generation buffers of one complete generation TP group, then slice and fuse
  per training rank.
* Zero redundancy (Section 5.3 last paragraph, Section 5.4, Table 2): a rank's own
  training shard is a subset of its generation partition; only the d_g-1 peers'
  pieces are "remote".

The paper is silent on tensor layouts.  Readings fixed here (listed in the design
notes of the repository):  rank r = dp*p*t + pp*t + tp;  first stage owns the
embedding, last stage owns the final norm and the untied LM head;  weights are
row-major [out, in];  the training shard stores Megatron-style fused tensors
  qkv   [(n_q+2*n_kv)/t * hd, h] : for each local KV group g (in order): the qpg
        query heads of g, then k_g, then v_g   (qpg = n_q/n_kv)
  gate_up [2F/t, h]              : gate rows of this rank, then up rows of this rank
and the generation buffer stores q, k, v, gate, up separately.  Byte layout of both
buffers: tensors in the order given by `TRAIN_LAYER_ORDER` / `GEN_LAYER_ORDER` below (embed first, final norm and head last), every tensor
start rounded up to 256 bytes, every rank region rounded up to 4096 bytes, regions
concatenated in rank order (generation: in the order of the materialised ranks).

parity pins: tests/test_oracle_*.py (paper's Figure 8 worked example, Table 2 closed
forms, brute-force element maps, round trip, overlap invariant, library-concat
special cases; the offload image by brute force over single elements, the Table 2
volume and hand-worked offsets).  The fused-QKV group order, the gate/up order and the stage that owns
embed/head are conventions of this repository, not of the paper: for them parity is
"unpinned by the paper" and pinned only by the hand-written fixtures in tests/golden.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Dict, List, Sequence, Tuple

import numpy as np

ELEM_BYTES = 2
TENSOR_ALIGN = 256
RANK_ALIGN = 4096

# order of tensors inside one layer, and around the layers
TRAIN_LAYER_ORDER = ("ln1", "qkv", "o", "ln2", "gate_up", "down")
GEN_LAYER_ORDER = ("ln1", "q", "k", "v", "o", "ln2", "gate", "up", "down")
# logical (unfused, unsharded) tensors
FULL_LAYER_NAMES = ("ln1", "wq", "wk", "wv", "wo", "ln2", "wg", "wu", "wd")
REPLICATED = ("ln1", "ln2", "lnf")

Fetch = Callable[[int, int], np.ndarray]  # (element offset, n elements) -> 1-D array


@dataclass(frozen=True)
class Model:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int


@dataclass(frozen=True)
class TrainLayout:
    pp: int
    tp: int
    dp: int = 1


@dataclass(frozen=True)
class GenLayout:
    pp: int
    tp: int
    grouping: str = "hybridflow"  # or "vanilla"


@dataclass(frozen=True)
class Entry:
    """One tensor inside one rank's region."""
    kind: str
    layer: int          # global layer index; -1 for embed / lnf / head
    rows: int
    cols: int
    offset: int         # ELEMENT offset from the start of the rank's region

    @property
    def n(self) -> int:
        return self.rows * self.cols


def _round_up(x: int, a: int) -> int:
    return (x + a - 1) // a * a


class ReshardOracle:
    def __init__(self, model: Model, train: TrainLayout, gen: GenLayout):
        m, tl, gl = model, train, gen
        for v in (*m.__dict__.values(), tl.pp, tl.tp, tl.dp, gl.pp, gl.tp):
            if not isinstance(v, int) or v <= 0:
                raise ValueError("all sizes must be positive integers")
        if gl.grouping not in ("hybridflow", "vanilla"):
            raise ValueError("unknown grouping")
        bad = []
        if tl.tp % gl.tp: bad.append("t % t_g")
        if tl.pp % gl.pp: bad.append("p % p_g")
        if m.n_layers % tl.pp: bad.append("L % p")
        if m.n_layers % gl.pp: bad.append("L % p_g")
        if m.vocab % tl.tp: bad.append("V % t")
        if m.ffn % tl.tp: bad.append("F % t")
        if m.n_q_heads % m.n_kv_heads: bad.append("n_q % n_kv")
        if m.n_kv_heads % tl.tp: bad.append("n_kv % t")
        if m.n_kv_heads % gl.tp: bad.append("n_kv % t_g")
        if bad:
            raise ValueError("not divisible: " + ", ".join(bad))
        self.m, self.tl, self.gl = m, tl, gl
        self.p, self.t, self.d = tl.pp, tl.tp, tl.dp
        self.pg, self.tg = gl.pp, gl.tp
        self.a = self.t // self.tg           # training TP shards per generation TP shard
        self.b = self.p // self.pg           # training stages per generation stage
        self.dg = self.a * self.b            # micro-DP size, d_g = p t / (p_g t_g)
        self.n_ranks = self.p * self.t * self.d
        self.qpg = m.n_q_heads // m.n_kv_heads
        self.lps = m.n_layers // self.p      # layers per training stage
        self.lpgs = m.n_layers // self.pg    # layers per generation stage
        # Replicated norms must be identical on all TP ranks of a stage; switch the
        # check off only to push rank tags or element indices through the same code.
        self.check_replicas = True
        self._memo: Dict[tuple, object] = {}  # tables only; never data

    # ------------------------------------------------------------------ groups
    def rank_of(self, dp: int, pp: int, tp: int) -> int:
        return dp * self.p * self.t + pp * self.t + tp

    def train_coords(self, r: int) -> Tuple[int, int, int]:
        """(dp, pp, tp) of rank r: TP fastest, then PP, DP at stride p*t."""
        pt = self.p * self.t
        return r // pt, (r % pt) // self.t, r % self.t

    def gen_coords(self, r: int) -> Tuple[int, int, int]:
        """(gpp, gtp, micro) of rank r in the generation stage."""
        dp, pp, tp = self.train_coords(r)
        if self.gl.grouping == "hybridflow":
            # generation TP / PP peers sit t/t_g resp. p/p_g training ranks apart, so
            # the generation index is the quotient and the micro-DP index the remainder
            return pp // self.b, tp // self.a, (pp % self.b) * self.a + tp % self.a
        i = pp * self.t + tp                 # position inside the replica
        return (i // self.tg) % self.pg, i % self.tg, i // (self.tg * self.pg)

    def _groups_by(self, keyfn) -> List[List[int]]:
        groups: Dict[tuple, List[int]] = {}
        for r in range(self.n_ranks):
            groups.setdefault(keyfn(r), []).append(r)
        return sorted(groups.values())

    def train_tp_groups(self):
        return self._groups_by(lambda r: self.train_coords(r)[:2])

    def train_pp_groups(self):
        return self._groups_by(lambda r: (self.train_coords(r)[0], self.train_coords(r)[2]))

    def train_dp_groups(self):
        return self._groups_by(lambda r: self.train_coords(r)[1:])

    def gen_tp_groups(self):
        return self._groups_by(lambda r: (self.train_coords(r)[0], self.gen_coords(r)[0], self.gen_coords(r)[2]))

    def gen_pp_groups(self):
        return self._groups_by(lambda r: (self.train_coords(r)[0], self.gen_coords(r)[1], self.gen_coords(r)[2]))

    def micro_dp_groups(self):
        return self._groups_by(lambda r: (self.train_coords(r)[0], self.gen_coords(r)[0], self.gen_coords(r)[1]))

    # ------------------------------------------------------------------ tables
    def _train_shape(self, kind: str) -> Tuple[int, int]:
        m, t = self.m, self.t
        return {
            "embed": (m.vocab // t, m.hidden),
            "head": (m.vocab // t, m.hidden),
            "ln1": (1, m.hidden), "ln2": (1, m.hidden), "lnf": (1, m.hidden),
            "qkv": ((m.n_q_heads + 2 * m.n_kv_heads) // t * m.head_dim, m.hidden),
            "o": (m.hidden, m.n_q_heads * m.head_dim // t),
            "gate_up": (2 * m.ffn // t, m.hidden),
            "down": (m.hidden, m.ffn // t),
        }[kind]

    def _gen_shape(self, kind: str) -> Tuple[int, int]:
        m, tg = self.m, self.tg
        return {
            "embed": (m.vocab // tg, m.hidden),
            "head": (m.vocab // tg, m.hidden),
            "ln1": (1, m.hidden), "ln2": (1, m.hidden), "lnf": (1, m.hidden),
            "q": (m.n_q_heads * m.head_dim // tg, m.hidden),
            "k": (m.n_kv_heads * m.head_dim // tg, m.hidden),
            "v": (m.n_kv_heads * m.head_dim // tg, m.hidden),
            "o": (m.hidden, m.n_q_heads * m.head_dim // tg),
            "gate": (m.ffn // tg, m.hidden),
            "up": (m.ffn // tg, m.hidden),
            "down": (m.hidden, m.ffn // tg),
        }[kind]

    @staticmethod
    def _lay_out(items) -> Tuple[List[Entry], int]:
        out, off = [], 0
        for kind, layer, (rows, cols) in items:
            off = _round_up(off, TENSOR_ALIGN // ELEM_BYTES)
            out.append(Entry(kind, layer, rows, cols, off))
            off += rows * cols
        return out, _round_up(off, RANK_ALIGN // ELEM_BYTES)

    def _table(self, first: bool, last: bool, layers: range, order, shape) -> Tuple[List[Entry], int]:
        items = []
        if first:
            items.append(("embed", -1, shape("embed")))
        for l in layers:
            for kind in order:
                items.append((kind, l, shape(kind)))
        if last:
            items.append(("lnf", -1, shape("lnf")))
            items.append(("head", -1, shape("head")))
        return self._lay_out(items)

    def train_table(self, r: int) -> Tuple[List[Entry], int]:
        """(entries, region size in elements) of rank r's training shard."""
        if ("tt", r) not in self._memo:
            _, pp, _ = self.train_coords(r)
            layers = range(pp * self.lps, (pp + 1) * self.lps)
            self._memo[("tt", r)] = self._table(pp == 0, pp == self.p - 1, layers, TRAIN_LAYER_ORDER, self._train_shape)
        return self._memo[("tt", r)]

    def gen_table(self, r: int) -> Tuple[List[Entry], int]:
        """(entries, region size in elements) of rank r's generation buffer."""
        if ("gt", r) not in self._memo:
            gpp, _, _ = self.gen_coords(r)
            layers = range(gpp * self.lpgs, (gpp + 1) * self.lpgs)
            self._memo[("gt", r)] = self._table(gpp == 0, gpp == self.pg - 1, layers, GEN_LAYER_ORDER, self._gen_shape)
        return self._memo[("gt", r)]

    def train_region_offsets(self) -> List[int]:
        """Element offset of every rank's region in train_buf, plus the total."""
        if "tro" not in self._memo:
            offs, off = [], 0
            for r in range(self.n_ranks):
                offs.append(off)
                off += self.train_table(r)[1]
            self._memo["tro"] = offs + [off]
        return self._memo["tro"]

    def gen_region_offsets(self, mat_ranks: Sequence[int]) -> List[int]:
        """Element offset of each materialised rank's region in gen_buf, plus total."""
        offs, off = [], 0
        for r in mat_ranks:
            offs.append(off)
            off += self.gen_table(r)[1]
        return offs + [off]

    def train_entry(self, r: int, kind: str, layer: int) -> Entry:
        if ("te", r) not in self._memo:
            self._memo[("te", r)] = {(e.kind, e.layer): e for e in self.train_table(r)[0]}
        return self._memo[("te", r)][(kind, layer)]

    def gen_entry(self, r: int, kind: str, layer: int) -> Entry:
        if ("ge", r) not in self._memo:
            self._memo[("ge", r)] = {(e.kind, e.layer): e for e in self.gen_table(r)[0]}
        return self._memo[("ge", r)][(kind, layer)]

    def input_regions(self, tensor_uid) -> List[Tuple[int, int, int]]:
        """(element offset in train_buf, n, uid) for the seeded generator.

        TP-sharded tensors get one stream per TP index; replicated norms use TP
        index 0 on every rank so that the copies are identical; the DP index is not
        part of the stream id, so DP replicas are identical too.
        """
        bases = self.train_region_offsets()
        regs = []
        for r in range(self.n_ranks):
            _, _, tp = self.train_coords(r)
            for e in self.train_table(r)[0]:
                uid = tensor_uid(e.kind, max(e.layer, 0), 0 if e.kind in REPLICATED else tp)
                regs.append((bases[r] + e.offset, e.n, uid))
        return regs

    # ----------------------------------------------- step 1: training -> generation
    def _stage_of(self, name: str, layer: int) -> int:
        if name == "embed":
            return 0
        if name in ("lnf", "head"):
            return self.p - 1
        return layer // self.lps

    def _train_tensor(self, fetch: Fetch, r: int, kind: str, layer: int) -> np.ndarray:
        e = self.train_entry(r, kind, layer)
        base = self.train_region_offsets()[r]
        return np.asarray(fetch(base + e.offset, e.n)).reshape(e.rows, e.cols)

    def full_from_train(self, fetch: Fetch, dp: int, name: str, layer: int, take_tp: int = 0) -> np.ndarray:
        """Rebuild one full logical tensor of replica `dp` from all t training shards.

        Replicated norms are read from TP index `take_tp` of the owning stage (a rank
        naturally uses the replica with its own TP index) and checked against all
        other TP ranks.
        """
        m, t = self.m, self.t
        pp = self._stage_of(name, layer)
        ranks = [self.rank_of(dp, pp, tp) for tp in range(t)]
        hd, qpg = m.head_dim, self.qpg
        if name in REPLICATED:
            copies = [self._train_tensor(fetch, r, name, layer) for r in ranks]
            if self.check_replicas:
                for c in copies:
                    if not np.array_equal(c, copies[take_tp]):
                        raise AssertionError(f"replicated tensor {name}[{layer}] differs across TP ranks")
            return copies[take_tp]
        if name in ("embed", "head"):
            return np.concatenate([self._train_tensor(fetch, r, name, layer) for r in ranks], axis=0)
        if name in ("wq", "wk", "wv"):
            lo, hi = {"wq": (0, qpg * hd), "wk": (qpg * hd, (qpg + 1) * hd), "wv": ((qpg + 1) * hd, (qpg + 2) * hd)}[name]
            parts = []
            for r in ranks:
                fused = self._train_tensor(fetch, r, "qkv", layer)
                per_group = fused.reshape(m.n_kv_heads // t, (qpg + 2) * hd, m.hidden)
                parts.append(per_group[:, lo:hi, :].reshape(-1, m.hidden))
            return np.concatenate(parts, axis=0)
        if name in ("wg", "wu"):
            fl = m.ffn // t
            sl = slice(0, fl) if name == "wg" else slice(fl, 2 * fl)
            return np.concatenate([self._train_tensor(fetch, r, "gate_up", layer)[sl] for r in ranks], axis=0)
        if name == "wo":
            return np.concatenate([self._train_tensor(fetch, r, "o", layer) for r in ranks], axis=1)
        if name == "wd":
            return np.concatenate([self._train_tensor(fetch, r, "down", layer) for r in ranks], axis=1)
        raise KeyError(name)

    _GEN_TO_FULL = {"embed": "embed", "head": "head", "ln1": "ln1", "ln2": "ln2", "lnf": "lnf",
                    "q": "wq", "k": "wk", "v": "wv", "o": "wo", "gate": "wg", "up": "wu", "down": "wd"}

    def gen_tensor(self, fetch: Fetch, r: int, kind: str, layer: int) -> np.ndarray:
        """One tensor of rank r's generation partition, from the training shards."""
        dp, _, tp = self.train_coords(r)
        _, gtp, _ = self.gen_coords(r)
        name = self._GEN_TO_FULL[kind]
        full = self.full_from_train(fetch, dp, name, layer, take_tp=tp)
        rows, cols = self._gen_shape(kind)
        if name in REPLICATED:
            return full
        if name in ("wo", "wd"):                      # row-parallel: split the input dim
            return np.ascontiguousarray(full[:, gtp * cols:(gtp + 1) * cols])
        return full[gtp * rows:(gtp + 1) * rows]      # column-parallel: split the output dim

    def reshard(self, train_buf: np.ndarray, gen_buf: np.ndarray, mat_ranks: Sequence[int]) -> np.ndarray:
        """Write the generation partition of every rank in `mat_ranks` into gen_buf.

        Both buffers are flat arrays with one item per bf16 element (any dtype, so the
        same code also transports element indices or rank tags).  Padding between
        tensors is left as it was.
        """
        fetch = lambda o, n: train_buf[o:o + n]
        bases = self.gen_region_offsets(mat_ranks)
        for i, r in enumerate(mat_ranks):
            for e in self.gen_table(r)[0]:
                val = self.gen_tensor(fetch, r, e.kind, e.layer)
                assert val.shape == (e.rows, e.cols)
                gen_buf[bases[i] + e.offset: bases[i] + e.offset + e.n] = val.reshape(-1)
        return gen_buf

    # ------------------- step 1 when the training weights live inside the generation buffers
    # Section 5.3 (last paragraph) and Section 5.4: under the HybridFlow grouping the training
    # weights of a GPU are a sub-part of its generation weights and are used in place, so the
    # all-gather of step 1 collects, from every micro-DP peer, the piece that peer trains --
    # out of the peer's generation buffer.  Same plain definition as above, with another
    # source: rebuild each full tensor from the pieces the training ranks hold INSIDE THEIR
    # GENERATION BUFFERS, then slice.
    def own_piece_from_gen(self, fetch_gen: Callable[[int, int, int], np.ndarray], q: int, name: str, layer: int) -> np.ndarray:
        """The part of full tensor `name` that rank q trains, read from q's generation buffer.

        fetch_gen(rank, element offset inside that rank's region, n) -> 1-D array.
        """
        if self.gl.grouping != "hybridflow":
            raise ValueError("only the HybridFlow grouping keeps the training shard inside the generation partition")
        _, _, tp = self.train_coords(q)
        _, gtp, _ = self.gen_coords(q)
        kind = {v: k for k, v in self._GEN_TO_FULL.items()}[name]
        e = self.gen_entry(q, kind, layer)
        held = np.asarray(fetch_gen(q, e.offset, e.n)).reshape(e.rows, e.cols)
        if name in REPLICATED:
            return held
        rows_full, cols_full = self.full_shape(name)
        if name in ("wo", "wd"):                       # split along the input dim
            per_t, per_g = cols_full // self.t, cols_full // self.tg
            lo = tp * per_t - gtp * per_g              # where the training columns start inside the generation columns
            assert 0 <= lo and lo + per_t <= per_g
            return held[:, lo:lo + per_t]
        per_t, per_g = rows_full // self.t, rows_full // self.tg
        lo = tp * per_t - gtp * per_g
        assert 0 <= lo and lo + per_t <= per_g
        return held[lo:lo + per_t]

    def full_from_own_views(self, fetch_gen, dp: int, name: str, layer: int, take_tp: int = 0) -> np.ndarray:
        """Rebuild one full logical tensor of replica `dp` from the pieces its t training ranks
        hold inside their generation buffers (norms: the copy of TP index `take_tp`)."""
        pp = self._stage_of(name, layer)
        ranks = [self.rank_of(dp, pp, tp) for tp in range(self.t)]
        if name in REPLICATED:
            return self.own_piece_from_gen(fetch_gen, ranks[take_tp], name, layer)
        axis = 1 if name in ("wo", "wd") else 0
        return np.concatenate([self.own_piece_from_gen(fetch_gen, q, name, layer) for q in ranks], axis=axis)

    def gather_in_place(self, gen_buf: np.ndarray, mat_ranks: Sequence[int]) -> np.ndarray:
        """Complete the generation buffers of `mat_ranks` (which hold their own pieces, and
        anything elsewhere) from each other: every tensor is rebuilt from the own views and
        sliced.  Needs the generation buffer of every training rank that owns a piece."""
        bases = self.gen_region_offsets(mat_ranks)
        pos = {r: i for i, r in enumerate(mat_ranks)}
        source = gen_buf.copy()                        # all reads see the state before the gather

        def fetch_gen(q, off, n):
            if q not in pos:
                raise KeyError(f"generation buffer of rank {q} is not materialised")
            return source[bases[pos[q]] + off: bases[pos[q]] + off + n]

        for i, r in enumerate(mat_ranks):
            dp, _, tp = self.train_coords(r)
            _, gtp, _ = self.gen_coords(r)
            for e in self.gen_table(r)[0]:
                name = self._GEN_TO_FULL[e.kind]
                full = self.full_from_own_views(fetch_gen, dp, name, e.layer, take_tp=tp)
                if name in REPLICATED:
                    val = full
                elif name in ("wo", "wd"):
                    val = full[:, gtp * e.cols:(gtp + 1) * e.cols]
                else:
                    val = full[gtp * e.rows:(gtp + 1) * e.rows]
                gen_buf[bases[i] + e.offset: bases[i] + e.offset + e.n] = np.ascontiguousarray(val).reshape(-1)
        return gen_buf

    # ----------------------------------------------- step 4: generation -> training
    def full_from_gen(self, fetch_gen: Callable[[int, int, int], np.ndarray], r: int, name: str, layer: int) -> np.ndarray:
        """Rebuild a full tensor from the generation TP group that rank r belongs to.

        fetch_gen(rank, element offset inside that rank's region, n) -> 1-D array.
        """
        dp, _, _ = self.train_coords(r)
        gpp, _, micro = self.gen_coords(r)
        group = [q for q in range(self.n_ranks)
                 if self.train_coords(q)[0] == dp and self.gen_coords(q)[0] == gpp and self.gen_coords(q)[2] == micro]
        group.sort(key=lambda q: self.gen_coords(q)[1])
        assert [self.gen_coords(q)[1] for q in group] == list(range(self.tg))
        kind = {v: k for k, v in self._GEN_TO_FULL.items()}[name]

        def piece(q):
            e = self.gen_entry(q, kind, layer)
            return np.asarray(fetch_gen(q, e.offset, e.n)).reshape(e.rows, e.cols)

        if name in REPLICATED:
            return piece(r)
        axis = 1 if name in ("wo", "wd") else 0
        return np.concatenate([piece(q) for q in group], axis=axis)

    def train_tensor_from_full(self, full: Callable[[str], np.ndarray], r: int, kind: str) -> np.ndarray:
        """Megatron-layout training tensor of rank r from full tensors (full(name))."""
        m, t = self.m, self.t
        _, _, tp = self.train_coords(r)
        rows, cols = self._train_shape(kind)
        hd, qpg = m.head_dim, self.qpg
        if kind in REPLICATED:
            return full(kind)
        if kind in ("embed", "head"):
            return full(kind)[tp * rows:(tp + 1) * rows]
        if kind == "o":
            return np.ascontiguousarray(full("wo")[:, tp * cols:(tp + 1) * cols])
        if kind == "down":
            return np.ascontiguousarray(full("wd")[:, tp * cols:(tp + 1) * cols])
        if kind == "gate_up":
            fl = m.ffn // t
            return np.concatenate([full("wg")[tp * fl:(tp + 1) * fl], full("wu")[tp * fl:(tp + 1) * fl]], axis=0)
        if kind == "qkv":
            wq, wk, wv = full("wq"), full("wk"), full("wv")
            blocks = []
            ng = m.n_kv_heads // t
            for j in range(ng):
                g = tp * ng + j
                blocks += [wq[g * qpg * hd:(g + 1) * qpg * hd], wk[g * hd:(g + 1) * hd], wv[g * hd:(g + 1) * hd]]
            return np.concatenate(blocks, axis=0)
        raise KeyError(kind)

    def reshard_back(self, gen_buf: np.ndarray, mat_ranks: Sequence[int], train_buf: np.ndarray,
                     ranks: Sequence[int] | None = None) -> np.ndarray:
        """Rewrite train_buf[r] for r in `ranks` (default: all materialised ranks).

        Needs the generation buffers of the whole generation TP group of each such
        rank to be present in gen_buf.
        """
        gbases = self.gen_region_offsets(mat_ranks)
        pos = {r: i for i, r in enumerate(mat_ranks)}

        def fetch_gen(q, off, n):
            if q not in pos:
                raise KeyError(f"generation buffer of rank {q} is not materialised")
            return gen_buf[gbases[pos[q]] + off: gbases[pos[q]] + off + n]

        tbases = self.train_region_offsets()
        for r in (mat_ranks if ranks is None else ranks):
            for e in self.train_table(r)[0]:
                val = self.train_tensor_from_full(
                    lambda name, _l=e.layer: self.full_from_gen(fetch_gen, r, name, _l), r, e.kind)
                assert val.shape == (e.rows, e.cols)
                train_buf[tbases[r] + e.offset: tbases[r] + e.offset + e.n] = val.reshape(-1)
        return train_buf

    # ------------------------------------------ element-by-element definitions
    # A second, deliberately dumb formulation: where does ONE element of a full
    # logical tensor live?  Scalar integer arithmetic only; used to pin the array
    # formulation above and to check single sampled elements at full model sizes.
    def full_shape(self, name: str) -> Tuple[int, int]:
        m = self.m
        return {
            "embed": (m.vocab, m.hidden), "head": (m.vocab, m.hidden),
            "ln1": (1, m.hidden), "ln2": (1, m.hidden), "lnf": (1, m.hidden),
            "wq": (m.n_q_heads * m.head_dim, m.hidden),
            "wk": (m.n_kv_heads * m.head_dim, m.hidden),
            "wv": (m.n_kv_heads * m.head_dim, m.hidden),
            "wo": (m.hidden, m.n_q_heads * m.head_dim),
            "wg": (m.ffn, m.hidden), "wu": (m.ffn, m.hidden), "wd": (m.hidden, m.ffn),
        }[name]

    def where_train(self, dp: int, name: str, layer: int, row: int, col: int) -> List[Tuple[int, int]]:
        """[(rank, element offset in train_buf)] of element (row, col) of a full tensor.

        One location for TP-sharded tensors, t locations for replicated norms.
        """
        m, t = self.m, self.t
        hd, qpg, h = m.head_dim, self.qpg, m.hidden
        pp = self._stage_of(name, layer)
        bases = self.train_region_offsets()

        def at(tp, kind, lrow, lcol):
            r = self.rank_of(dp, pp, tp)
            e = self.train_entry(r, kind, layer)
            assert 0 <= lrow < e.rows and 0 <= lcol < e.cols
            return (r, bases[r] + e.offset + lrow * e.cols + lcol)

        if name in REPLICATED:
            return [at(tp, name, 0, col) for tp in range(t)]
        if name in ("embed", "head"):
            per = m.vocab // t
            return [at(row // per, name, row % per, col)]
        if name == "wq":
            head, within = divmod(row, hd)
            g, jq = divmod(head, qpg)             # KV group and query index in it
            tp, j = divmod(g, m.n_kv_heads // t)
            return [at(tp, "qkv", j * (qpg + 2) * hd + jq * hd + within, col)]
        if name in ("wk", "wv"):
            g, within = divmod(row, hd)
            tp, j = divmod(g, m.n_kv_heads // t)
            slot = qpg if name == "wk" else qpg + 1
            return [at(tp, "qkv", j * (qpg + 2) * hd + slot * hd + within, col)]
        if name in ("wg", "wu"):
            per = m.ffn // t
            return [at(row // per, "gate_up", (0 if name == "wg" else per) + row % per, col)]
        if name == "wo":
            per = m.n_q_heads * hd // t
            return [at(col // per, "o", row, col % per)]
        if name == "wd":
            per = m.ffn // t
            return [at(col // per, "down", row, col % per)]
        raise KeyError(name)

    def where_gen(self, dp: int, name: str, layer: int, row: int, col: int) -> List[Tuple[int, int]]:
        """[(rank, element offset inside that rank's generation region)] for every
        rank of replica `dp` whose generation partition holds the element."""
        m, tg = self.m, self.tg
        if name == "embed":
            gpp = 0
        elif name in ("lnf", "head"):
            gpp = self.pg - 1
        else:
            gpp = layer // self.lpgs
        kind = {v: k for k, v in self._GEN_TO_FULL.items()}[name]
        rows, cols = self._gen_shape(kind)
        if name in REPLICATED:
            gtp, lrow, lcol = None, 0, col
        elif name in ("wo", "wd"):
            gtp, lrow, lcol = col // cols, row, col % cols
        else:
            gtp, lrow, lcol = row // rows, row % rows, col
        out = []
        for r in range(self.n_ranks):
            if self.train_coords(r)[0] != dp:
                continue
            rgpp, rgtp, _ = self.gen_coords(r)
            if rgpp == gpp and (gtp is None or rgtp == gtp):
                e = self.gen_entry(r, kind, layer)
                out.append((r, e.offset + lrow * e.cols + lcol))
        return out

    def full_tensor_names(self) -> List[Tuple[str, int]]:
        names = [("embed", -1)]
        for l in range(self.m.n_layers):
            names += [(n, l) for n in FULL_LAYER_NAMES]
        return names + [("lnf", -1), ("head", -1)]

    # ---------------------------------- step 3: all-gather of results in a micro-DP group
    def micro_dp_members(self, r: int) -> List[int]:
        """Ranks of r's micro-DP group, ordered by micro-DP index."""
        dp = self.train_coords(r)[0]
        gpp, gtp, _ = self.gen_coords(r)
        members = [q for q in range(self.n_ranks)
                   if self.train_coords(q)[0] == dp and self.gen_coords(q)[:2] == (gpp, gtp)]
        return sorted(members, key=lambda q: self.gen_coords(q)[2])

    def gather_responses(self, resp_in: np.ndarray) -> np.ndarray:
        """Section 5.2 step 3.  resp_in[r] = results of rank r's generation replica (any
        trailing shape); returns out[r] = concatenation, along a new leading axis of
        length d_g, of the results of r's micro-DP group members in micro-DP order: what an
        all-gather inside the group leaves on every member."""
        assert resp_in.shape[0] == self.n_ranks
        return np.stack([np.stack([resp_in[q] for q in self.micro_dp_members(r)]) for r in range(self.n_ranks)])

    # ---------------------- offload image of the remote pieces (Section 7, "Implementation")
    # The generation copy of the weights leaves the GPU while the model trains.  What a
    # rank has to move is what the transition gathered for it: the elements of its
    # generation partition that do not come from its own training shard (Section 5.3: the
    # own shard is reused in place).  Reading of this repository (the paper gives no
    # format): the image lists, for every materialised rank in buffer order and every
    # generation tensor in table order, the remote elements in row-major order; a rank's
    # part starts at a multiple of RANK_ALIGN bytes, a tensor's part at a multiple of
    # TENSOR_ALIGN bytes, tensors without remote elements take no space.
    def owner_tags(self, mat_ranks: Sequence[int]) -> np.ndarray:
        """gen_buf-shaped int32 array: the rank whose training shard supplies each element
        (-1 for padding), obtained by pushing rank tags through the concat/slice code."""
        offs = self.train_region_offsets()
        tags = np.empty(offs[-1], dtype=np.int32)
        for q in range(self.n_ranks):
            tags[offs[q]:offs[q + 1]] = q
        saved, self.check_replicas = self.check_replicas, False   # norm copies carry different tags
        try:
            return self.reshard(tags, np.full(self.gen_region_offsets(mat_ranks)[-1], -1, dtype=np.int32), mat_ranks)
        finally:
            self.check_replicas = saved

    def remote_layout(self, mat_ranks: Sequence[int]):
        """(parts, rank_offsets, total): parts = [(rank, Entry, image element offset, mask)]
        with mask = bool array over the tensor's elements (row-major), True = remote."""
        tags = self.owner_tags(mat_ranks)
        bases = self.gen_region_offsets(mat_ranks)
        parts, rank_offsets, off = [], [], 0
        for i, r in enumerate(mat_ranks):
            off = _round_up(off, RANK_ALIGN // ELEM_BYTES)
            rank_offsets.append(off)
            for e in self.gen_table(r)[0]:
                mask = tags[bases[i] + e.offset: bases[i] + e.offset + e.n] != r
                n = int(mask.sum())
                if n == 0:
                    continue
                off = _round_up(off, TENSOR_ALIGN // ELEM_BYTES)
                parts.append((r, e, off, mask))
                off += n
        return parts, rank_offsets, _round_up(off, RANK_ALIGN // ELEM_BYTES)

    def pack_remote(self, gen_buf: np.ndarray, mat_ranks: Sequence[int], image: np.ndarray) -> np.ndarray:
        """Offload: copy the remote elements of gen_buf into `image` (gaps left as they are)."""
        parts, _, total = self.remote_layout(mat_ranks)
        assert image.shape[0] >= total
        bases = dict(zip(mat_ranks, self.gen_region_offsets(mat_ranks)))
        for r, e, off, mask in parts:
            vals = gen_buf[bases[r] + e.offset: bases[r] + e.offset + e.n][mask]
            image[off:off + vals.shape[0]] = vals
        return image

    def unpack_remote(self, image: np.ndarray, gen_buf: np.ndarray, mat_ranks: Sequence[int]) -> np.ndarray:
        """Reload: put the image's elements back; own pieces and padding are not written."""
        parts, _, _ = self.remote_layout(mat_ranks)
        bases = dict(zip(mat_ranks, self.gen_region_offsets(mat_ranks)))
        for r, e, off, mask in parts:
            view = gen_buf[bases[r] + e.offset: bases[r] + e.offset + e.n]
            view[mask] = image[off:off + int(mask.sum())]
        return gen_buf

    # ------------------------------------------------- Table 2 closed forms (bytes)
    def model_bytes(self) -> int:
        return ELEM_BYTES * sum(int(np.prod(self.full_shape(n))) for n, _ in self.full_tensor_names())

    def table2(self, M: int) -> Dict[str, Dict[str, float]]:
        """Section 5.4, Table 2, evaluated for this configuration and a model of M bytes."""
        t, p, d, tg, pg = self.t, self.p, self.d, self.tg, self.pg
        return {
            "ds_chat": {"comm": (t * p * d - 1) / (t * p * d) * M, "peak": M, "redundancy": M / (t * p * d)},
            "hybridflow_v": {"comm": (t * p - 1) / (t * p) * M, "peak": M, "redundancy": M / (t * p)},
            "hybridflow": {"comm": (t * p - tg * pg) / (tg * pg * t * p) * M, "peak": M / (tg * pg), "redundancy": 0.0},
        }

    def full_coords_of_gen(self, r: int, kind: str, lrow: int, lcol: int) -> Tuple[str, int, int]:
        """(full tensor name, row, col) of element (lrow, lcol) of rank r's generation
        tensor `kind`: the slice rule of the generation partition read backwards."""
        _, gtp, _ = self.gen_coords(r)
        name = self._GEN_TO_FULL[kind]
        rows, cols = self._gen_shape(kind)
        if name in REPLICATED:
            return name, 0, lcol
        if name in ("wo", "wd"):
            return name, lrow, gtp * cols + lcol
        return name, gtp * rows + lrow, lcol
