"""The benchmark workloads (synthetic stand-ins for the paper's five-dataset mixture): five of growing size, and a
sixth with the model shape the paper trains (4 layers of 866 hidden units, heads of three layers of 889 units, local
batch of 128 structures: section "Numerical Results").

Each entry restates one workload: how many graphs, how atoms are drawn, cutoff, hidden width H,
number of message-passing layers L, GEMM operand type and number of sources S. The datasets the paper
trains on are not available; these batches only take their shape (small CHNO(+F,S) molecules for the
organic sets, periodic crystals over most of the periodic table for the inorganic sets, five sources,
batches of about a hundred graphs).
"""
from __future__ import annotations

import numpy as np

from .structures import Batch, concat_graphs, make_crystal, make_cubic_bulk, make_molecule

CONFIGS = {
    "cfg1": dict(desc="32 non-periodic CHNO molecules, 4-20 atoms, 6 A box", rc=5.0, H=64, L=3,
                 dtype="f32", S=1, seed=0),
    "cfg2": dict(desc="128 molecules, 10-60 atoms, 0.08 atoms/A^3, 5 sources", rc=5.0, H=128, L=4,
                 dtype="f32", S=5, seed=0),
    "cfg3": dict(desc="64 periodic triclinic crystals, 8-120 atoms", rc=6.0, H=256, L=4,
                 dtype="bf16", S=1, seed=0),
    "cfg4": dict(desc="mixed 5-source batch, ~40k atoms / ~1.2M edges", rc=5.0, H=256, L=6,
                 dtype="bf16", S=5, seed=0),
    "cfg5": dict(desc="4 periodic cubic cells of 20,000 atoms at 0.1 atoms/A^3", rc=6.0, H=128, L=3,
                 dtype="f32", S=1, seed=0),
    "cfg6": dict(desc="the paper's model shape: 128 mixed 5-source structures, H=866, heads 3 x 889", rc=5.0, H=866,
                 L=4, dtype="bf16", S=5, seed=0, Hh=889, D=3),
}

_MOL_Z2 = (1, 6, 7, 8, 9, 16)


def _molecule_cfg2(rng, n):
    side = (n / 0.08) ** (1.0 / 3.0)
    return make_molecule(rng, n, side, 0.9, _MOL_Z2)


def _gen_cfg1(rng) -> Batch:
    graphs = []
    for _ in range(32):
        n = int(rng.integers(4, 21))
        graphs.append(make_molecule(rng, n, 6.0, 0.9, (1, 6, 7, 8), (0.5, 0.3, 0.1, 0.1)))
    return concat_graphs(graphs)


def _gen_cfg2(rng) -> Batch:
    graphs = []
    for _ in range(128):
        n = int(rng.integers(10, 61))
        graphs.append(_molecule_cfg2(rng, n))
    src = rng.integers(0, 5, size=128).astype(np.int32)
    return concat_graphs(graphs, src)


def _gen_cfg3(rng) -> Batch:
    graphs = []
    for _ in range(64):
        n = int(rng.integers(8, 121))
        graphs.append(make_crystal(rng, n, 4.0, 15.0, 1.2, 1, 94))
    return concat_graphs(graphs)


def _gen_cfg4(rng, n_target=40000, crystal_density_cap=0.085) -> Batch:
    graphs, src = [], []
    total = 0
    while total < n_target:
        s = int(rng.integers(0, 5))
        if s <= 2:
            n = int(rng.integers(5, 61))
            graphs.append(_molecule_cfg2(rng, n))
        else:
            n = int(rng.integers(8, 201))
            graphs.append(make_crystal(rng, n, 4.0, 15.0, 1.2, 1, 94,
                                       max_density=crystal_density_cap))
        src.append(s)
        total += n
    return concat_graphs(graphs, np.asarray(src, dtype=np.int32),
                         meta=dict(crystal_density_cap=crystal_density_cap))


def _gen_cfg6(rng, n_graphs=128, crystal_density_cap=0.085) -> Batch:
    """One local batch of the paper's size, every structure drawn like those of the mixed batch of config 4."""
    graphs, src = [], []
    for _ in range(n_graphs):
        s = int(rng.integers(0, 5))
        if s <= 2:
            graphs.append(_molecule_cfg2(rng, int(rng.integers(5, 61))))
        else:
            graphs.append(make_crystal(rng, int(rng.integers(8, 201)), 4.0, 15.0, 1.2, 1, 94,
                                       max_density=crystal_density_cap))
        src.append(s)
    return concat_graphs(graphs, np.asarray(src, dtype=np.int32), meta=dict(crystal_density_cap=crystal_density_cap))


def _gen_cfg5(rng, n_graphs=4, n_atoms=20000) -> Batch:
    graphs = [make_cubic_bulk(rng, n_atoms, 0.1, 1.0, 1, 30) for _ in range(n_graphs)]
    return concat_graphs(graphs)


_GEN = {"cfg1": _gen_cfg1, "cfg2": _gen_cfg2, "cfg3": _gen_cfg3, "cfg4": _gen_cfg4, "cfg5": _gen_cfg5,
        "cfg6": _gen_cfg6}


def make_config(name: str, seed: int | None = None, **overrides) -> tuple[Batch, dict]:
    """Return (batch, hyper-parameters) of one named workload. Structure stream = child 0 of the seed."""
    hp = dict(CONFIGS[name])
    if seed is not None:
        hp["seed"] = seed
    ss = np.random.SeedSequence(hp["seed"])
    rng = np.random.default_rng(ss.spawn(3)[0])
    batch = _GEN[name](rng, **overrides)
    hp["name"] = name
    return batch, hp


def small_mixed_batch(seed: int, n_mol=3, n_cry=3, S=3, mol_atoms=(3, 14), cry_atoms=(2, 10),
                      cry_len=(3.0, 7.0), dmin=0.9) -> Batch:
    """A tiny batch for tests: a few molecules and a few small triclinic crystals, interleaved,
    sources drawn uniformly. Small cells make several periodic images (and self-images) per pair."""
    rng = np.random.default_rng(seed)
    graphs = []
    kinds = [0] * n_mol + [1] * n_cry
    rng.shuffle(kinds)
    for kind in kinds:
        if kind == 0:
            n = int(rng.integers(mol_atoms[0], mol_atoms[1] + 1))
            side = (n / 0.05) ** (1.0 / 3.0)
            graphs.append(make_molecule(rng, n, side, dmin, _MOL_Z2))
        else:
            n = int(rng.integers(cry_atoms[0], cry_atoms[1] + 1))
            graphs.append(make_crystal(rng, n, cry_len[0], cry_len[1], dmin, 1, 94, max_density=0.15))
    src = rng.integers(0, S, size=len(graphs)).astype(np.int32)
    return concat_graphs(graphs, src)
