"""The calibrated configurations of a model as a file: what persists between the offline
determination (Alg. 1, once per model) and inference.  Plain JSON, written and read here;
no arithmetic of the method."""
from __future__ import annotations

import json

import numpy as np

FORMAT = "tca-calibration-1"


def save_calibration(path: str, prm, cal: dict, M: int, sigma: float, tau: float, L_cal: int) -> None:
    """cal: the dict returned by tca_calibrate_layers (or tca_calibrate_budgets, taken as one layer)."""
    p_star = np.asarray(cal["p_star"], np.float64)
    cand = np.asarray(cal["cand_idx"])
    fb = np.asarray(cal["fallback"])
    if p_star.ndim == 2:
        p_star, cand, fb = p_star[None], cand[None], fb[None]
    doc = {
        "format": FORMAT,
        "n_q_heads": prm.n_q_heads, "n_kv_heads": prm.n_kv_heads, "head_dim": prm.head_dim,
        "block": prm.block, "window": prm.window, "alpha": prm.alpha, "metric": prm.metric, "share": prm.share,
        "candidates": M, "sigma": sigma, "tau": tau, "calibration_tokens": L_cal,
        "n_layers": int(p_star.shape[0]), "n_selection_heads": int(p_star.shape[1]),
        # doubles survive JSON exactly through repr (Python writes the shortest string that round-trips)
        "p_star": p_star.tolist(), "cand_idx": cand.astype(int).tolist(), "fallback": fb.astype(int).tolist(),
    }
    with open(path, "w") as f:
        json.dump(doc, f)


def load_calibration(path: str, prm=None) -> dict:
    """Returns dict(p_star [layers,Hs,nk] float64, cand_idx, fallback, and the recorded settings).
    With prm given, refuses a file calibrated for another layer shape, block size or selection mode."""
    with open(path) as f:
        doc = json.load(f)
    if doc.get("format") != FORMAT:
        raise ValueError(f"{path}: not a {FORMAT} file")
    if prm is not None:
        for key in ("n_q_heads", "n_kv_heads", "head_dim", "block", "share", "metric"):
            if doc[key] != getattr(prm, key):
                raise ValueError(f"{path}: calibrated with {key}={doc[key]}, the layer has {getattr(prm, key)}")
    doc["p_star"] = np.asarray(doc["p_star"], np.float64)
    doc["cand_idx"] = np.asarray(doc["cand_idx"], np.int32)
    doc["fallback"] = np.asarray(doc["fallback"], np.int32)
    if doc["p_star"].shape[:2] != (doc["n_layers"], doc["n_selection_heads"]):
        raise ValueError(f"{path}: p_star has shape {doc['p_star'].shape}")
    return doc
