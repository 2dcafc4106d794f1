"""Plain CPU oracle for type-directed array redistribution (arXiv 2112.01075).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the
benchmark's CPU-baseline leg; never by the product path.  Shares no code,
tables or helpers with the HIP library or its planner.

Everything is written out from the paper's definitions, slowly and literally:

  * distributed types, meta-functions            -- Fig. "Meshes, distributed types, and meta-functions"
  * base-offset maps D[[.]] and T[[.]]            -- Fig. "Base offset maps"
  * well-formedness, validity                     -- Fig. "Well-formedness rules", Sec. 2.5
  * the four collectives (typing + data effect)   -- Fig. "Typing collective operations", Def. 4.3, Sec. 7.1
  * low-level collectives on device assignments   -- Fig. "Semantics of low-level collective operations"
  * cost, height, normal form                     -- Fig. cost model, Def. 4.4, Def. 4.5
  * shortest-path searches (weak and strict)      -- Sec. 7.2, Sec. 6.2
  * naive redistribution                          -- Eq. (2)

Conventions fixed where the paper is silent (each one is pinned by a test):
  - a local tile is a dense row-major array;
  - shard index = row-major index of the mesh coordinate, axes in
    declaration order, last axis fastest;
  - an axis of composite size k splits into prime axes "x.0", "x.1", ...
    (factors ascending, minor to major) replacing x in place in every axis
    list; the decomposed mesh declares them major-most first so that the
    shard order does not change.

Pinning status: every function here is pinned by tests/test_oracle_*.py
(worked examples printed in the paper, Lemmas 4.1/4.2 as properties, printed
costs, closed-form NumPy special cases, brute force); shard_of, the
one-shard-at-a-time form of distribute that the GPU tests take their inputs
and expected tiles from, is pinned in tests/test_oracle_types.py against
distribute, against the linear index of an iota array and against the
printed offset example of Sec. 2.1.  Nothing is unpinned.
"""
from __future__ import annotations

import heapq
import itertools
import re
from collections import Counter, namedtuple
from math import prod

import numpy as np

# A distributed dimension  c{axes}n  (axes minor-to-major, fastest first).
Dim = namedtuple("Dim", ["c", "axes", "n"])


# --------------------------------------------------------------------------
# syntax helpers
# --------------------------------------------------------------------------
def parse_type(text):
    """Parse "[8{x,y}32, 128]" (quotes and ":k" size suffixes tolerated)."""
    body = text.strip()
    if not (body.startswith("[") and body.endswith("]")):
        raise ValueError("type must be bracketed: %r" % text)
    body = body[1:-1]
    dims, depth, cur = [], 0, ""
    for ch in body:
        if ch == "{":
            depth += 1
        if ch == "}":
            depth -= 1
        if ch == "," and depth == 0:
            dims.append(cur)
            cur = ""
        else:
            cur += ch
    if cur.strip():
        dims.append(cur)
    out = []
    for d in dims:
        d = d.strip().replace('"', "").replace("'", "")
        m = re.fullmatch(r"(\d+)\s*\{([^}]*)\}\s*(\d+)", d)
        if m:
            axes = tuple(a.strip().split(":")[0].strip() for a in m.group(2).split(",") if a.strip())
            out.append(Dim(int(m.group(1)), axes, int(m.group(3))))
        else:
            n = int(d)
            out.append(Dim(n, (), n))
    return tuple(out)


def format_type(typ):
    parts = []
    for d in typ:
        parts.append(str(d.n) if not d.axes and d.c == d.n else "%d{%s}%d" % (d.c, ",".join(d.axes), d.n))
    return "[" + ", ".join(parts) + "]"


# --------------------------------------------------------------------------
# meta-functions (Fig. "Meshes, distributed types, and meta-functions")
# --------------------------------------------------------------------------
def axes_of(typ):
    return [x for d in typ for x in d.axes]


def rank(typ):
    return len(typ)


def globaltype(typ):
    return tuple(d.n for d in typ)


def globalsize(typ):
    return prod(d.n for d in typ)


def localtype(typ):
    return tuple(d.c for d in typ)


def localsize(typ):
    return prod(d.c for d in typ)


def mesh_size(mesh):
    return prod(mesh.values())


# --------------------------------------------------------------------------
# well-formedness and validity
# --------------------------------------------------------------------------
def wf_dim(mesh, dim):
    """Rule wf-dim: axes exist, are pairwise distinct, c * prod(k) == n."""
    if dim.c < 1 or dim.n < 1:
        return False
    if any(x not in mesh for x in dim.axes):
        return False
    if len(set(dim.axes)) != len(dim.axes):
        return False
    return dim.c * prod(mesh[x] for x in dim.axes) == dim.n


def wf_type(mesh, typ):
    """Rule wf-type: every dim well-formed; axis lists pairwise disjoint."""
    if not all(wf_dim(mesh, d) for d in typ):
        return False
    allax = axes_of(typ)
    return len(set(allax)) == len(allax)


def valid_redistribution(t1, t2):
    """Sec. 2.5: valid iff the global array types agree."""
    return globaltype(t1) == globaltype(t2)


# --------------------------------------------------------------------------
# base-offset maps (Fig. "Base offset maps")
# --------------------------------------------------------------------------
def D(dim, mesh, coord):
    """D[[c{}c]] = 0 ;  D[[c{x,xs}n]](i) = c*i_x + D[[(c*k_x){xs}n]](i)."""
    if not dim.axes:
        if dim.c != dim.n:
            raise ValueError("ill-formed base case %r" % (dim,))
        return 0
    x = dim.axes[0]
    return dim.c * coord[x] + D(Dim(dim.c * mesh[x], dim.axes[1:], dim.n), mesh, coord)


def T(typ, mesh, coord):
    return tuple(D(d, mesh, coord) for d in typ)


def mesh_coords(mesh):
    """All mesh coordinates in shard order (declaration order, last axis fastest)."""
    names = list(mesh.keys())
    return [dict(zip(names, idx)) for idx in itertools.product(*[range(mesh[x]) for x in names])]


def offset_table(typ, mesh):
    """Base offset of every shard, in shard order."""
    return [T(typ, mesh, c) for c in mesh_coords(mesh)]


# --------------------------------------------------------------------------
# distribute / undistribute (Sec. 4.1, Lemma 4.2)
# --------------------------------------------------------------------------
def _box(off, shape):
    return tuple(slice(o, o + s) for o, s in zip(off, shape))


def distribute(G, mesh, typ):
    """Shard k holds G[T(k) : T(k) + localtype]."""
    if tuple(G.shape) != globaltype(typ):
        raise ValueError("global shape mismatch")
    if not wf_type(mesh, typ):
        raise ValueError("ill-formed type")
    shape = localtype(typ)
    return [np.ascontiguousarray(G[_box(off, shape)]) for off in offset_table(typ, mesh)]


def shard_of(G, mesh, typ, k):
    """Shard k alone (same definition as distribute; for arrays too large to shard at once)."""
    shape = localtype(typ)
    return np.ascontiguousarray(G[_box(T(typ, mesh, mesh_coords(mesh)[k]), shape)])


def undistribute(shards, mesh, typ):
    """Inverse of distribute; checks replicas agree and the tiles cover G."""
    shape = localtype(typ)
    G = np.zeros(globaltype(typ), dtype=shards[0].dtype)
    seen = np.zeros(globaltype(typ), dtype=bool)
    for off, tile in zip(offset_table(typ, mesh), shards):
        if tuple(tile.shape) != shape:
            raise ValueError("tile shape mismatch")
        b = _box(off, shape)
        if seen[b].any():
            # tiles either coincide or are disjoint; replicas must agree bit for bit
            if not seen[b].all() or np.ascontiguousarray(G[b]).tobytes() != np.ascontiguousarray(tile).tobytes():
                raise ValueError("replicas disagree at %r" % (off,))
        G[b] = tile
        seen[b] = True
    if not seen.all():
        raise ValueError("tiles do not cover the global array")
    return G


# --------------------------------------------------------------------------
# typing rules of the collectives, multi-axis form (Fig. typing, Sec. 7.1)
# --------------------------------------------------------------------------
def _axes_size(mesh, xs):
    return prod(mesh[x] for x in xs)


def rule_allgather(mesh, typ, i, k=1):
    """Remove the k minor-most axes of dim i; tile grows by their product."""
    d = typ[i]
    if k < 1 or len(d.axes) < k:
        raise ValueError("allgather: dim %d has fewer than %d axes" % (i, k))
    f = _axes_size(mesh, d.axes[:k])
    new = Dim(d.c * f, d.axes[k:], d.n)
    return typ[:i] + (new,) + typ[i + 1:]


def rule_dynslice(mesh, typ, i, xs):
    """Prepend the unused axes xs to dim i; tile shrinks by their product."""
    xs = tuple(xs)
    if not xs:
        raise ValueError("dynslice: no axis")
    used = set(axes_of(typ))
    if any(x not in mesh for x in xs) or len(set(xs)) != len(xs) or any(x in used for x in xs):
        raise ValueError("dynslice: axis unknown, repeated or already in use")
    d = typ[i]
    f = _axes_size(mesh, xs)
    if d.c % f:
        raise ValueError("dynslice: local size not divisible")
    new = Dim(d.c // f, xs + d.axes, d.n)
    return typ[:i] + (new,) + typ[i + 1:]


def rule_alltoall(mesh, typ, i, j, k=1):
    """Move the k minor-most axes of dim i to the front of dim j."""
    if i == j:
        raise ValueError("alltoall: i == j")
    di, dj = typ[i], typ[j]
    if k < 1 or len(di.axes) < k:
        raise ValueError("alltoall: dim %d has fewer than %d axes" % (i, k))
    xs = di.axes[:k]
    f = _axes_size(mesh, xs)
    if dj.c % f:
        raise ValueError("alltoall: c_j mod n != 0")
    out = list(typ)
    out[i] = Dim(di.c * f, di.axes[k:], di.n)
    out[j] = Dim(dj.c // f, xs + dj.axes, dj.n)
    return tuple(out)


def rule_allpermute_ok(t1, t2):
    return localtype(t1) == localtype(t2) and globaltype(t1) == globaltype(t2)


# --------------------------------------------------------------------------
# the collectives acting on data: one NumPy tile per mesh coordinate
# (Def. 4.3: the typing rule fixes the effect; chunk order follows i_x)
# --------------------------------------------------------------------------
def _mixed_radix(mesh, xs, coord):
    """Value of the coordinates on xs, first axis fastest."""
    v, w = 0, 1
    for x in xs:
        v += coord[x] * w
        w *= mesh[x]
    return v


def allgather(shards, mesh, typ, i, k=1):
    new_t = rule_allgather(mesh, typ, i, k)
    xs = typ[i].axes[:k]
    coords = mesh_coords(mesh)
    out = [None] * len(coords)
    groups = {}
    for idx, c in enumerate(coords):
        key = tuple(v for x, v in c.items() if x not in xs)
        groups.setdefault(key, []).append(idx)
    for members in groups.values():
        members = sorted(members, key=lambda m: _mixed_radix(mesh, xs, coords[m]))
        cat = np.concatenate([shards[m] for m in members], axis=i)
        for m in members:
            out[m] = cat.copy()
    return out, new_t


def dynslice(shards, mesh, typ, i, xs):
    new_t = rule_dynslice(mesh, typ, i, xs)
    cprime = new_t[i].c
    out = []
    for c, tile in zip(mesh_coords(mesh), shards):
        m = _mixed_radix(mesh, xs, c)
        sl = [slice(None)] * tile.ndim
        sl[i] = slice(m * cprime, (m + 1) * cprime)
        out.append(np.ascontiguousarray(tile[tuple(sl)]))
    return out, new_t


def alltoall(shards, mesh, typ, i, j, k=1):
    """alltoall(i,j) == allgather(i) then dynslice(j, same axes) (Peak Lemma, case 3)."""
    new_t = rule_alltoall(mesh, typ, i, j, k)
    xs = typ[i].axes[:k]
    g, tg = allgather(shards, mesh, typ, i, k)
    out, tt = dynslice(g, mesh, tg, j, xs)
    assert tt == new_t
    return out, new_t


def allpermute(shards, mesh, t1, t2):
    """T[[t2]] = T[[t1]] o pi (Lemma 5.1): each device takes the tile of a holder."""
    if not rule_allpermute_ok(t1, t2):
        raise ValueError("allpermute: local or global types differ")
    tab1 = offset_table(t1, mesh)
    holder = {}
    for idx, off in enumerate(tab1):
        holder.setdefault(off, idx)
    out = []
    for off in offset_table(t2, mesh):
        out.append(shards[holder[off]].copy())
    return out, t2


def naive_redistribute(shards, mesh, t1, t2):
    """Eq. (2): gather every dim fully, then slice every dim as t2 demands.

    Returns (shards, list of intermediate types)."""
    types = [t1]
    cur, typ = shards, t1
    for i in range(len(typ)):
        if typ[i].axes:
            cur, typ = allgather(cur, mesh, typ, i, len(typ[i].axes))
            types.append(typ)
    for i in range(len(t2)):
        if t2[i].axes:
            cur, typ = dynslice(cur, mesh, typ, i, t2[i].axes)
            types.append(typ)
    assert typ == t2
    return cur, types


def redistribute_by_definition(shards, mesh, t1, t2):
    """The plain definition of the result: slices of the global array."""
    if not valid_redistribution(t1, t2):
        raise ValueError("global types differ")
    return distribute(undistribute(shards, mesh, t1), mesh, t2)


# --------------------------------------------------------------------------
# cost, height, normal form
# --------------------------------------------------------------------------
def step_cost(kind, L_before, L_after):
    """Fig. cost model (elements per device)."""
    if kind == "allpermute":
        return L_before
    if kind == "dynslice":
        return 0
    if kind == "allgather":
        return L_after
    if kind == "alltoall":
        return L_before
    raise ValueError(kind)


def sequence_cost(kinds, localsizes):
    """kinds[k] takes localsizes[k] to localsizes[k+1]."""
    assert len(localsizes) == len(kinds) + 1
    return sum(step_cost(k, localsizes[n], localsizes[n + 1]) for n, k in enumerate(kinds))


def height(localsizes):
    """Def. 4.4."""
    return max(localsizes)


_NF = re.compile(r"^(d)*(t|p)*(g)*$")
_NF_LETTER = {"dynslice": "d", "alltoall": "t", "allpermute": "p", "allgather": "g"}


def is_normal_form(kinds):
    """Def. 4.5: dynslice* {alltoall|allpermute}* allgather*."""
    return bool(_NF.match("".join(_NF_LETTER[k] for k in kinds)))


# --------------------------------------------------------------------------
# prime decomposition of the mesh (Sec. 3, Principle 1)
# --------------------------------------------------------------------------
def prime_factors(k):
    out, p = [], 2
    while k > 1:
        while k % p == 0:
            out.append(p)
            k //= p
        p += 1
    return out


def decompose(mesh, *types):
    """Equivalent problem over prime axes: x:k -> x.0, x.1, ... (minor to major in
    every dimension's axis list).  The new mesh declares x's factors major-most
    first, so the shard order (last declared axis fastest) is unchanged."""
    new_mesh, sub = {}, {}
    for x, k in mesh.items():
        fs = prime_factors(k)
        names = ["%s.%d" % (x, t) for t in range(len(fs))]
        sub[x] = tuple(names)
        for nm, p in reversed(list(zip(names, fs))):
            new_mesh[nm] = p
    new_types = []
    for typ in types:
        new_types.append(tuple(Dim(d.c, tuple(y for x in d.axes for y in sub[x]), d.n) for d in typ))
    return (new_mesh, *new_types)


# --------------------------------------------------------------------------
# low-level collectives on device assignments
# (Fig. "Semantics of low-level collective operations"): physical device d
# holds the tile at offs[d]; only this table is physically meaningful.
# --------------------------------------------------------------------------
class DeviceState:
    """shape = local tile shape, offs[d] = base offset held by physical device d,
    tiles[d] = the data (or None when only bookkeeping is replayed)."""

    def __init__(self, gshape, shape, offs, tiles=None):
        self.gshape = tuple(gshape)
        self.shape = tuple(shape)
        self.offs = [tuple(o) for o in offs]
        self.tiles = tiles

    @property
    def ndev(self):
        return len(self.offs)

    def localsize(self):
        return prod(self.shape)

    def check_weak_type(self):
        """offs must be (a permutation of) T[[tau]] for a well-formed tau with this
        local type: all base offsets occur, each equally often."""
        for s, n in zip(self.shape, self.gshape):
            if n % s:
                raise AssertionError("tile does not divide global dim")
        for o in self.offs:
            if any(v % s or v < 0 or v >= n for v, s, n in zip(o, self.shape, self.gshape)):
                raise AssertionError("offset %r is not a base offset" % (o,))
        cnt = Counter(self.offs)
        ntiles = prod(n // s for s, n in zip(self.shape, self.gshape))
        if len(cnt) != ntiles or len(set(cnt.values())) != 1:
            raise AssertionError("offset table is not a balanced cover")

    def check_data(self, G):
        for o, t in zip(self.offs, self.tiles):
            if t.shape != self.shape or G[_box(o, self.shape)].tobytes() != np.ascontiguousarray(t).tobytes():
                raise AssertionError("device tile differs from the global slice at %r" % (o,))


def _check_groups(state, i, groups, f):
    seen = set()
    c = state.shape[i]
    for g in groups:
        if len(g) != f:
            raise AssertionError("group size %d != %d" % (len(g), f))
        base = state.offs[g[0]]
        if base[i] % (c * f):
            raise AssertionError("group does not start an aligned super-tile")
        for r, d in enumerate(g):
            if d in seen:
                raise AssertionError("device in two groups")
            seen.add(d)
            o = state.offs[d]
            if any(o[t] != base[t] for t in range(len(o)) if t != i) or o[i] != base[i] + r * c:
                raise AssertionError("group members are not the adjacent tiles in rank order")
    if len(seen) != state.ndev:
        raise AssertionError("groups do not partition the devices")


def ll_allgather(state, i, groups):
    """groups: lists of physical devices in rank order; each group ends with the
    concatenation along dim i of its members' tiles."""
    f = len(groups[0])
    _check_groups(state, i, groups, f)
    shape = list(state.shape)
    shape[i] *= f
    offs = list(state.offs)
    tiles = [None] * state.ndev if state.tiles is not None else None
    for g in groups:
        base = state.offs[g[0]]
        cat = np.concatenate([state.tiles[d] for d in g], axis=i) if tiles is not None else None
        for d in g:
            offs[d] = base
            if tiles is not None:
                tiles[d] = cat.copy()
    return DeviceState(state.gshape, shape, offs, tiles)


def ll_alltoall(state, i, j, groups):
    """Group member of rank q ends with chunk q (along dim j) of the group's
    concatenation along dim i."""
    if i == j:
        raise AssertionError("alltoall: i == j")
    f = len(groups[0])
    _check_groups(state, i, groups, f)
    if state.shape[j] % f:
        raise AssertionError("alltoall: c_j mod n != 0")
    cj = state.shape[j] // f
    shape = list(state.shape)
    shape[i] *= f
    shape[j] = cj
    offs = list(state.offs)
    tiles = [None] * state.ndev if state.tiles is not None else None
    for g in groups:
        base = list(state.offs[g[0]])
        cat = np.concatenate([state.tiles[d] for d in g], axis=i) if tiles is not None else None
        for q, d in enumerate(g):
            o = list(base)
            o[j] = base[j] + q * cj
            offs[d] = tuple(o)
            if tiles is not None:
                sl = [slice(None)] * len(shape)
                sl[j] = slice(q * cj, (q + 1) * cj)
                tiles[d] = np.ascontiguousarray(cat[tuple(sl)])
    return DeviceState(state.gshape, shape, offs, tiles)


def ll_dynslice(state, i, f, chunk):
    """Device d keeps chunk[d] (of f) along dim i.  Legal iff the result is again a
    balanced cover (some relabelling of replicas realises it through a fresh axis)."""
    if state.shape[i] % f:
        raise AssertionError("dynslice: local size not divisible")
    c = state.shape[i] // f
    shape = list(state.shape)
    shape[i] = c
    offs, tiles = [], ([] if state.tiles is not None else None)
    for d in range(state.ndev):
        m = chunk[d]
        if not 0 <= m < f:
            raise AssertionError("chunk index out of range")
        o = list(state.offs[d])
        o[i] += m * c
        offs.append(tuple(o))
        if tiles is not None:
            sl = [slice(None)] * len(shape)
            sl[i] = slice(m * c, (m + 1) * c)
            tiles.append(np.ascontiguousarray(state.tiles[d][tuple(sl)]))
    out = DeviceState(state.gshape, shape, offs, tiles)
    out.check_weak_type()
    return out


def ll_allpermute(state, src):
    """Device d receives the whole tile of device src[d]; src must be a bijection."""
    if sorted(src) != list(range(state.ndev)):
        raise AssertionError("allpermute: not a bijection")
    offs = [state.offs[s] for s in src]
    tiles = [state.tiles[s].copy() for s in src] if state.tiles is not None else None
    return DeviceState(state.gshape, state.shape, offs, tiles)


# --------------------------------------------------------------------------
# searches
# --------------------------------------------------------------------------
def _divisors_from(counter):
    """All products of sub-multisets of a prime multiset (as a Counter), > 1."""
    outs = {1}
    for p, m in counter.items():
        outs = {o * p ** e for o in outs for e in range(m + 1)}
    outs.discard(1)
    return sorted(outs)


def _prime_counter(n):
    return Counter(prime_factors(n))


def weak_search(gshape, mesh_sizes, c1, c2, normal_form=False, step_latency=0):
    """Sec. 7.2: shortest path over weak types (= local types, global type fixed).

    step_latency (elements; 0 = the paper's cost model): added to the weight of every step
    that communicates (allgather, alltoall).  This is the latency-aware cost the paper's
    discussion of the adversarial table names as future work (Sec. 8); the returned cost
    then includes step_latency per communicating step.

    With normal_form=True only label strings dynslice* alltoall* allgather* are
    allowed (Def. 4.5 without permutes); by the lemma on normal forms of weak
    sequences this cannot cost more.

    Nodes: local types whose partition factors' primes fit in the mesh's prime
    multiset and whose local size is within max(L1, L2).  Edges: multi-axis weak
    collectives, weighted by the cost model.  Returns (cost, [(kind,i,j,f,localtype)])."""
    gshape, c1, c2 = tuple(gshape), tuple(c1), tuple(c2)
    mesh_primes = Counter()
    for k in mesh_sizes:
        mesh_primes.update(prime_factors(k))
    bound = max(prod(c1), prod(c2))
    r = len(gshape)

    def used(c):
        u = Counter()
        for t in range(r):
            u.update(prime_factors(gshape[t] // c[t]))
        return u

    def realisable(c):
        u = used(c)
        return all(u[p] <= mesh_primes[p] for p in u)

    assert realisable(c1) and realisable(c2)

    def edges(c):
        L = prod(c)
        u = used(c)
        free = Counter({p: mesh_primes[p] - u[p] for p in mesh_primes if mesh_primes[p] - u[p] > 0})
        for i in range(r):
            for f in _divisors_from(free):                      # dynslice
                if c[i] % f == 0:
                    yield ("dynslice", i, -1, f, c[:i] + (c[i] // f,) + c[i + 1:], 0)
            for f in _divisors_from(_prime_counter(gshape[i] // c[i])):
                if L * f <= bound:                              # allgather
                    yield ("allgather", i, -1, f, c[:i] + (c[i] * f,) + c[i + 1:], L * f + step_latency)
                for j in range(r):                              # alltoall
                    if j != i and c[j] % f == 0:
                        n = list(c)
                        n[i] *= f
                        n[j] //= f
                        yield ("alltoall", i, j, f, tuple(n), L + step_latency)

    phase_of = {"dynslice": 0, "alltoall": 1, "allgather": 2}
    start = (c1, 0)
    dist = {start: 0}
    prev = {}
    pq = [(0, 0, start)]
    tick = 1
    goal = None
    while pq:
        dcur, _, node = heapq.heappop(pq)
        if dcur > dist.get(node, float("inf")):
            continue
        c, ph = node
        if c == c2:
            goal = node
            break
        for kind, i, j, f, nc, w in edges(c):
            nph = 0
            if normal_form:
                nph = phase_of[kind]
                if nph < ph:
                    continue
            nn = (nc, nph)
            nd = dcur + w
            if nd < dist.get(nn, float("inf")):
                dist[nn] = nd
                prev[nn] = (node, (kind, i, j, f, nc))
                heapq.heappush(pq, (nd, tick, nn))
                tick += 1
    if goal is None:
        return None, None
    path, node = [], goal
    while node != start:
        node, e = prev[node]
        path.append(e)
    return dist[goal], path[::-1]


def all_wf_types(mesh, gshape):
    """Every well-formed syntactic type over mesh with this global type."""
    names = list(mesh.keys())
    r = len(gshape)
    out = []
    for assign in itertools.product(range(-1, r), repeat=len(names)):
        per_dim = [[x for x, a in zip(names, assign) if a == t] for t in range(r)]
        if any(gshape[t] % prod(mesh[x] for x in per_dim[t]) for t in range(r)):
            continue
        for orders in itertools.product(*[list(itertools.permutations(p)) for p in per_dim]):
            out.append(tuple(Dim(gshape[t] // prod(mesh[x] for x in orders[t]), tuple(orders[t]), gshape[t])
                             for t in range(r)))
    return out


def strict_search(mesh, t1, t2):
    """Memory-constrained optimal-cost problem of Sec. 6.2 by brute force over
    SYNTACTIC types: strict multi-axis collectives plus allpermute edges between
    types of equal local type; nodes bounded by max(L1, L2).
    Returns (cost, [(kind, type_after)])."""
    assert wf_type(mesh, t1) and wf_type(mesh, t2) and valid_redistribution(t1, t2)
    bound = max(localsize(t1), localsize(t2))
    by_local = {}
    for t in all_wf_types(mesh, globaltype(t1)):
        by_local.setdefault(localtype(t), []).append(t)

    def edges(t):
        L = localsize(t)
        used = set(axes_of(t))
        free = [x for x in mesh if x not in used]
        r = len(t)
        for i in range(r):
            for k in range(1, len(t[i].axes) + 1):
                nt = rule_allgather(mesh, t, i, k)
                if localsize(nt) <= bound:
                    yield "allgather", nt, localsize(nt)
                for j in range(r):
                    if j != i and t[j].c % _axes_size(mesh, t[i].axes[:k]) == 0:
                        yield "alltoall", rule_alltoall(mesh, t, i, j, k), L
            for k in range(1, len(free) + 1):
                for xs in itertools.permutations(free, k):
                    if t[i].c % _axes_size(mesh, xs) == 0:
                        yield "dynslice", rule_dynslice(mesh, t, i, xs), 0
        for nt in by_local[localtype(t)]:
            if nt != t:
                yield "allpermute", nt, L

    dist = {t1: 0}
    prev = {}
    pq = [(0, 0, t1)]
    tick = 1
    while pq:
        dcur, _, t = heapq.heappop(pq)
        if dcur > dist.get(t, float("inf")):
            continue
        if t == t2:
            break
        for kind, nt, w in edges(t):
            nd = dcur + w
            if nd < dist.get(nt, float("inf")):
                dist[nt] = nd
                prev[nt] = (t, (kind, nt))
                heapq.heappush(pq, (nd, tick, nt))
                tick += 1
    if t2 not in dist:
        return None, None
    path, t = [], t2
    while t != t1:
        t, e = prev[t]
        path.append(e)
    return dist[t2], path[::-1]
