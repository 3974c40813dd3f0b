"""Seeded synthetic clusters for the scheduler tests (inputs only: no cost-model arithmetic here).
Shapes follow the paper's testbeds (Sec. 5.2): nodes of one GPU generation each, fast links inside a
node (450 / 300 GB/s), a 25 GB/s fabric between nodes; device numbers are in the range of H100 / A100 / A800
data sheets."""
import numpy as np

KINDS = {  # dense bf16 FLOP/s, HBM bytes/s, HBM bytes, intra-node link bytes/s
    "h100": (989e12, 3.35e12, 80e9, 450e9),
    "a100": (312e12, 2.0e12, 80e9, 300e9),
    "a800": (312e12, 1.9e12, 40e9, 200e9),
}


def cluster_arrays(nodes, inter_bw=25e9, alpha_intra=5e-6, alpha_inter=2e-5, m_static=20e9, jitter_seed=None):
    """nodes: list of (kind, count).  Returns dict of python lists / nested lists."""
    kinds, node_of = [], []
    for i, (kind, cnt) in enumerate(nodes):
        kinds += [kind] * cnt
        node_of += [i] * cnt
    n = len(kinds)
    rng = np.random.default_rng(jitter_seed) if jitter_seed is not None else None
    jit = (lambda: float(rng.uniform(0.9, 1.1))) if rng is not None else (lambda: 1.0)
    c = [KINDS[k][0] * jit() for k in kinds]
    b = [KINDS[k][1] * jit() for k in kinds]
    m = [KINDS[k][2] for k in kinds]
    ms = [m_static] * n
    bw = [[0.0] * n for _ in range(n)]
    al = [[0.0] * n for _ in range(n)]
    for i in range(n):
        for j in range(n):
            if i == j:
                bw[i][j] = 1e30
            elif node_of[i] == node_of[j]:
                bw[i][j] = KINDS[kinds[i]][3]
                al[i][j] = alpha_intra
            else:
                bw[i][j] = inter_bw
                al[i][j] = alpha_inter
    return dict(c=c, b=b, m=m, m_static=ms, alpha=al, bw=bw)


def model_args(l_tot=131072, batch=1, hidden=4096, head_dim=128, n_heads=32, dtype_bytes=2):
    return dict(l_tot=l_tot, batch=batch, hidden=hidden, head_dim=head_dim, n_heads=n_heads, dtype_bytes=dtype_bytes)
