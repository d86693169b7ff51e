"""Index permutations between the paper's notation (NCHW activations, OIHW filters, linear
features flattened as (a, i, j)) and the library's memory layout (NHWC, KRSC / ARSK,
features flattened as (i, j, a)).  Pure re-indexing on numpy arrays: no arithmetic.
"""
from __future__ import annotations

import numpy as np


def act_to_lib(x):          # [B,C,H,W] -> [B,H,W,C]
    return np.ascontiguousarray(np.transpose(x, (0, 2, 3, 1)))


def act_from_lib(x):        # [B,H,W,C] -> [B,C,H,W]
    return np.ascontiguousarray(np.transpose(x, (0, 3, 1, 2)))


def filt_to_lib(w):         # [O,I,R,S] -> [O,R,S,I]
    return np.ascontiguousarray(np.transpose(w, (0, 2, 3, 1)))


def filt_from_lib(w):       # [O,R,S,I] -> [O,I,R,S]
    return np.ascontiguousarray(np.transpose(w, (0, 3, 1, 2)))


def fc_to_lib(wf, A, oh, ow):    # [Cls, (a,i,j)] -> [Cls, (i,j,a)]
    cls = wf.shape[0]
    return np.ascontiguousarray(wf.reshape(cls, A, oh, ow).transpose(0, 2, 3, 1).reshape(cls, -1))


def fc_from_lib(wf, A, oh, ow):  # [Cls, (i,j,a)] -> [Cls, (a,i,j)]
    cls = wf.shape[0]
    return np.ascontiguousarray(wf.reshape(cls, oh, ow, A).transpose(0, 3, 1, 2).reshape(cls, -1))


def params_to_lib(p: dict, A, oh=2, ow=2) -> dict:
    """dict W,b,Wp,Wa,ba,Wf,bf in paper notation -> library layout (None entries kept)."""
    return {
        "W": filt_to_lib(p["W"]), "b": np.ascontiguousarray(p["b"]),
        "Wp": None if p.get("Wp") is None else np.ascontiguousarray(p["Wp"]),
        "Wa": filt_to_lib(p["Wa"]), "ba": np.ascontiguousarray(p["ba"]),
        "Wf": fc_to_lib(p["Wf"], A, oh, ow), "bf": np.ascontiguousarray(p["bf"]),
    }


def params_from_lib(p: dict, A, oh=2, ow=2) -> dict:
    return {
        "W": filt_from_lib(p["W"]), "b": p["b"],
        "Wp": p.get("Wp"),
        "Wa": filt_from_lib(p["Wa"]), "ba": p["ba"],
        "Wf": fc_from_lib(p["Wf"], A, oh, ow), "bf": p["bf"],
    }
