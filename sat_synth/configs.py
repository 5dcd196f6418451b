"""Workload configurations.

Each entry mirrors the published shape statistics (node count, edge count,
feature width, class count) of one dataset row of the paper's dataset table;
the graphs themselves are seeded synthetic stand-ins, never the datasets.
"""

CONFIGS = {
    # toy case the oracle finishes in well under a second
    "tiny": dict(
        kind="sbm", N=4096, n_comm=2, n_parts=2, part=0,
        intra_deg=7.0, cross_deg=1.0,          # expected neighbours per node
        dims=[64, 32, 8], noise_std=0.01, tau=2, d_s=32, seed=0,
    ),
    # ogbn-arxiv-shaped: 169,343 nodes / 2.3 M edges / 128 features / 40 classes
    "medium": dict(
        kind="chung_lu", N=170_000, n_parts=4, part=0, mean_deg=13.0,
        gamma=2.1, cut=0.15, dims=[128, 256, 256, 40], noise_std=0.05,
        tau=2, d_s=64, seed=0,
    ),
    # Reddit-shaped: 232,965 nodes / 602 features / 41 classes, very high degree
    "dense": dict(
        kind="sbm", N=233_000, n_comm=50, n_parts=8, part=0,
        mean_deg=490.0, cut=0.25, dims=[602, 256, 41], noise_std=0.05,
        tau=2, d_s=64, seed=0,
    ),
    # ogbn-products-shaped: 2,449,029 nodes / 123.7 M edges / 100 features / 47 classes
    "large": dict(
        kind="chung_lu", N=2_450_000, n_parts=8, part=0, mean_deg=50.0,
        gamma=2.3, cut=0.20, dims=[100, 256, 256, 47], noise_std=0.05,
        tau=2, d_s=64, seed=0,
    ),
    # ogbn-papers100M-shaped (128 features / 172 classes, mean degree 29, bf16
    # storage) at 1/32 of its node count: one partition of 8 holds 434 k nodes
    "scale_small": dict(
        kind="chung_lu", N=3_470_000, n_parts=8, part=0, mean_deg=29.0,
        gamma=2.2, cut=0.20, dims=[128, 256, 256, 172], noise_std=0.05,
        tau=2, d_s=64, seed=0, dtype="bf16",
    ),
    # ogbn-papers100M-shaped at full size: 111 M nodes, 8 partitions, only partition 0's
    # rows are drawn (13.9 M local nodes, about 400 M CSR entries); no cut fraction is
    # published for it, 10 % is assumed; history tables hold local + halo rows only
    "scale": dict(
        kind="chung_lu_rows", N=111_000_000, n_parts=8, part=0, mean_deg=29.0,
        gamma=2.2, cut=0.10, dims=[128, 256, 256, 172], noise_std=0.05,
        tau=2, d_s=64, seed=0, dtype="bf16", tables="relabelled", device_inputs=True,
    ),
    # the same recipe at 1/64 of the node count (CPU tests of the generator)
    "scale_rows_small": dict(
        kind="chung_lu_rows", N=1_734_375, n_parts=8, part=0, mean_deg=29.0,
        gamma=2.2, cut=0.10, dims=[128, 256, 256, 172], noise_std=0.05,
        tau=2, d_s=64, seed=0, dtype="bf16", tables="relabelled", device_inputs=True,
    ),
}


def get_config(name):
    cfg = dict(CONFIGS[name])
    cfg["name"] = name
    return cfg
