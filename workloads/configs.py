"""The benchmark/parity configurations: shapes, mask recipe and seeds.

C1..C5 follow the five workload descriptions of the build's baseline file; C0d / C0c are the all-ones and
causal masks of the paper's Appendix C.  `small_variant` gives a reduced-size instance of the same mask family
that a CPU oracle finishes in seconds."""
import numpy as np
from . import masks
from .qkv import make_qkv

BASE_SEED = 1234

CONFIGS = {
    "C1": dict(B=1, H=2, N=256, d=64, Mb=1, family="random_blocks"),
    "C2": dict(B=4, H=16, N=4096, d=64, Mb=4, family="packed"),
    "C3": dict(B=8, H=32, N=1280, d=128, Mb=1, family="tree"),
    "C4": dict(B=1, H=16, N=16384, d=64, Mb=1, family="longctx"),
    "C5": dict(B=1, H=8, N=32768, d=64, Mb=1, family="graph"),
    "C0d": dict(B=4, H=16, N=4096, d=64, Mb=1, family="all_ones"),
    "C0c": dict(B=4, H=16, N=4096, d=64, Mb=1, family="causal"),
    "C0d128": dict(B=2, H=32, N=8192, d=128, Mb=1, family="all_ones"),
    "C0c128": dict(B=2, H=32, N=8192, d=128, Mb=1, family="causal"),
    # further mask families of the paper's evaluation (Sec. 5: ALPACA "Input-Bidirectional" packing; Longformer
    # "Windowed" and "Dilated" masks), at the shapes of the neighbouring configurations
    "C2b": dict(B=4, H=16, N=4096, d=64, Mb=4, family="packed_bidir"),
    "C4w": dict(B=1, H=16, N=16384, d=64, Mb=1, family="window"),
    "C4d": dict(B=1, H=16, N=16384, d=64, Mb=1, family="dilated"),
    # tree verification at decode time: only the 256 candidate-tree tokens are queries (Nq), the keys are the 1024-token
    # prefix plus the tree (N): the last Nq rows of the mask of C3
    "C3q": dict(B=8, H=32, N=1280, d=128, Mb=1, family="tree", Nq=256),
    # the same for a single sequence against a 16384-token cache: 64 work-groups of 128 queries, far fewer than the
    # chip has CUs, each with 260 tiles to walk
    "C3qL": dict(B=1, H=32, N=16640, d=128, Mb=1, family="tree", Nq=256),
    # the graph of C5 as it arrives, with scrambled node labels: the reordering is part of the measured pipeline
    "C5g": dict(B=1, H=8, N=32768, d=64, Mb=1, family="graph_scrambled", gpu_reorder=True),
}
_IDS = {k: i for i, k in enumerate(CONFIGS)}


def make_mask(family: str, N: int, Mb: int, seed: int) -> np.ndarray:
    if family == "random_blocks":
        return masks.random_blocks(N, seed)
    if family == "packed":
        hi = min(1024, max(16, N // 4))
        mu = 5.3 if N >= 4096 else np.log(max(20.0, N / 20.0))
        return masks.packed_sequences(N, Mb, seed, mu=mu, hi=hi)
    if family == "packed_bidir":     # the first 40 % of every packed sequence (its "input") attends in both directions
        hi = min(1024, max(16, N // 4))
        mu = 5.3 if N >= 4096 else np.log(max(20.0, N / 20.0))
        return masks.packed_sequences(N, Mb, seed, bidirectional_prefix=0.4, mu=mu, hi=hi)
    if family == "window":           # +-256 keys, as the window of the long-context configuration
        return masks.sliding_window(N, 256 if N >= 16384 else max(32, N // 32))
    if family == "dilated":          # 256 keys on each side, every second position: every block of the band is partial
        return masks.dilated_window(N, 256 if N >= 16384 else max(32, N // 32), 2)
    if family == "tree":
        tree = 256 if N >= 1280 else max(16, N // 5)
        return masks.tree_verification(N - tree, masks.random_subtree([10, 5, 3, 2], tree, seed))
    if family == "longctx":
        if N >= 16384:
            return masks.longctx_sparse(N, seed)
        return masks.longctx_sparse(N, seed, window=max(64, N // 32 * 2), n_global=min(64, N // 16), n_rand=2)
    if family == "graph":
        if N >= 32768:
            return masks.graph_mask(N, seed)
        f = N / 32768.0
        return masks.graph_mask(N, seed, xm=max(2.0, 84.0 * f * 4), cap=max(16, int(2000 * f * 4)))
    if family == "graph_scrambled":
        if N >= 32768:
            return masks.graph_mask(N, seed, reorder="none")
        f = N / 32768.0
        return masks.graph_mask(N, seed, reorder="none", xm=max(2.0, 84.0 * f * 4), cap=max(16, int(2000 * f * 4)))
    if family == "all_ones":
        return masks.all_ones(N)
    if family == "causal":
        return masks.causal(N)
    raise ValueError(family)


def make_config(name: str, with_qkv: bool = True, **override):
    """Returns dict(shape keys..., mask=uint8 [Mb,N,N], q/k/v = uint16 bf16 bit patterns [B,H,N,d])."""
    cfg = dict(CONFIGS[name])
    cfg.update(override)
    seed = BASE_SEED + _IDS[name]
    cfg["name"] = name
    cfg["seed"] = seed
    cfg["mask"] = make_mask(cfg["family"], cfg["N"], cfg["Mb"], seed)
    if with_qkv:
        cfg["q"], cfg["k"], cfg["v"] = make_qkv(cfg["B"], cfg["H"], cfg["N"], cfg["d"], seed + 100)
    if "Nq" in cfg:   # the last Nq tokens are the queries: mask [Mb, Nq, N], q [B, H, Nq, d]
        cfg["mask"] = np.ascontiguousarray(cfg["mask"][:, cfg["N"] - cfg["Nq"]:])
        if with_qkv:
            cfg["q"] = np.ascontiguousarray(cfg["q"][:, :, cfg["N"] - cfg["Nq"]:])
    return cfg


def small_variant(name: str, N: int, B: int = None, H: int = None, with_qkv: bool = True):
    """Same family, reduced N (and optionally B, H) so the dense fp64 oracle runs in seconds."""
    base = CONFIGS[name]
    B = base["B"] if B is None else B
    Mb = B if base["Mb"] > 1 else 1
    return make_config(name, with_qkv=with_qkv, N=N, B=B, H=base["H"] if H is None else H, Mb=Mb)
