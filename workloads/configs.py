"""The five benchmark configurations, with every value they leave open frozen here.

Keys: n, d, graph ("ring" | "reg4" | "hopring"), model ("lsq" | "logreg" |
"synth" | "mlp"), K events, M minibatch, rows per worker, gamma, lambda,
staleness law (tau_mode "uniform" with T_max, or "geometric" with per-class
(num, den) and cap T_max), worker weights (update frequencies p_i), seeds.
``small`` entries are reduced shapes of the same structure for tests.
"""
from __future__ import annotations

import copy

CONFIGS = {
    # 1: n=8 ring, least squares d=1024, N=1024 rows ~N(0,1), M=32, gamma=0.01, K=2000, tau~U{0..3}
    1: dict(name="cfg1_lsq_ring8", n=8, d=1024, graph="ring", model="lsq", K=2000, M=32,
            rows=1024, gamma=0.01, lam=0.0, tau_mode="uniform", T_max=3, seed=0,
            feature_var=1.0, noise=0.1),
    # 2: n=64 ring, logistic d=65536, lambda=1e-4, 4096 rows ~N(0,1/d), M=128, K=20000, tau~U{0..8}
    #    (gamma is not given by the configuration.  With |a| ~ 1 a step changes the margins of its
    #    own minibatch by about gamma/(2M) and those of the mean model by gamma/(2Mn): gamma = 64
    #    moves the local margins by 0.25 per step; 20000 events lower the loss 0.693 -> ~0.66,
    #    gamma >= 2048 diverges, gamma = 0.5 does not move at all)
    2: dict(name="cfg2_logreg_ring64", n=64, d=65536, graph="ring", model="logreg", K=20000,
            M=128, rows=4096, gamma=64.0, lam=1e-4, tau_mode="uniform", T_max=8, seed=0,
            noise=0.1),
    # 3: n=128 ring, ResNet-50-sized flat vector d=25.6M, synthetic g ~ N(0, 1e-3) (variance),
    #    K=100000, tau~U{0..16}; gamma = 0.1 (the paper's ResNet base learning rate, Sec. 5.2)
    3: dict(name="cfg3_synth_ring128", n=128, d=25_600_000, graph="ring", model="synth",
            K=100_000, M=0, rows=0, gamma=0.1, lam=0.0, tau_mode="uniform", T_max=16, seed=0,
            synth_std=0.0316227766016838),
    # 4: n=16 random 4-regular, MLP 784-1024-10, bf16 weights + fp32 master, 8192 samples,
    #    M=64, K=20000; tau and gamma not given: U{0..4}, 0.05
    4: dict(name="cfg4_mlp_reg4_16", n=16, d=784 * 1024 + 1024 + 1024 * 10 + 10, graph="reg4",
            model="mlp", K=20000, M=64, rows=8192, gamma=0.05, lam=0.0, tau_mode="uniform",
            T_max=4, seed=0, mlp=(784, 1024, 10)),
    # 5: n=32 random 4-regular, least squares d=4M (2^22), 4 workers 10x slower:
    #    p_i proportional to speed (weights 10 / 1), geometric staleness mean 2 (fast) and
    #    20 (slow), capped at 128; rows=64, M=8, features ~N(0,1/d); gamma not given: 4.0
    #    (rows have unit norm, so a step removes gamma/M = 1/2 of its minibatch residual;
    #    10000 events lower the loss 0.50 -> 0.15; gamma = 1 and 8 are stable as well)
    5: dict(name="cfg5_lsq_reg4_32_hetero", n=32, d=4 * 1024 * 1024, graph="reg4", model="lsq",
            K=50000, M=8, rows=64, gamma=4.0, lam=0.0, tau_mode="geometric", T_max=128, seed=0,
            n_slow=4, weight_fast=10, weight_slow=1, tau_fast=(2, 3), tau_slow=(20, 21),
            feature_var_inv_d=True, noise=0.1),
}


def get_config(idx: int, **overrides):
    cfg = copy.deepcopy(CONFIGS[idx])
    cfg.update(overrides)
    return cfg
