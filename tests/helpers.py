"""Glue used by tests only: turns a workload table into the oracle's NetSpec."""
import numpy as np

from oracle import alexnet_oracle as O


def oracle_spec(wl: dict, batch: int, seed: int = 0) -> O.NetSpec:
    n, k, a, b = wl["lrn"]
    return O.NetSpec(
        batch=batch, in_c=wl["in_c"], crop_h=wl["crop"], crop_w=wl["crop"], raw_h=wl["raw"], raw_w=wl["raw"],
        conv=[O.ConvSpec(co, kk, st, pd, g, bool(l), bool(p)) for (co, kk, st, pd, g, l, p) in wl["conv"]],
        fc=list(wl["fc"]), lrn_n=n, lrn_k=k, lrn_alpha=a, lrn_beta=b, dropout_p=wl["dropout_p"],
        lr=wl["lr"], momentum=wl["momentum"], weight_decay=wl["weight_decay"], seed=seed)


def to64(d):
    return {k: np.asarray(v, np.float64) for k, v in d.items()}


def rel_l2(a, b):
    a = np.asarray(a, np.float64).ravel()
    b = np.asarray(b, np.float64).ravel()
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a - b))
