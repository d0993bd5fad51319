"""Helpers for the GPU parity tests: run the HIP path and the oracle on the same seeded inputs."""
import numpy as np

import workloads as W
from oracle import zo
from oracle.precision import Precision, JitterPrecision  # noqa: F401  (re-exported for the tests)


def make_bundle(w, b_std=0.0, wseed=1234, lseed=99, tseed=2345):
    return dict(w=w, layout=W.lora_layout(w), frozen=W.make_frozen_weights(w, wseed),
                masters=W.make_lora_masters(w, lseed, b_std=b_std),
                tokens=W.make_tokens(w, tseed), labels=W.make_labels(w, tseed))


def gpu_model(b, **kw):
    import paper_2409_15520_amd as M
    return M.ZoModel(b["w"], b["frozen"], b["masters"], **kw)


def gpu_steps(b, n_steps, seed=3456, model=None, first_step=0):
    """Returns (losses[n_steps, 2q], g[n_steps, q], masters after the last step)."""
    import torch
    m = model or gpu_model(b)
    tok = torch.from_numpy(b["tokens"]).to(m.device)
    lab = torch.from_numpy(b["labels"]).to(m.device)
    L, G = [], []
    for s in range(first_step, first_step + n_steps):
        m.regen_noise(seed, s)
        L.append(m.forward_perturbed(tok, lab).cpu().numpy().astype(np.float64))
        G.append(m.zo_update().cpu().numpy().astype(np.float64))
    torch.cuda.synchronize()
    return np.array(L), np.array(G), m.masters.cpu().numpy()


def oracle_steps(b, n_steps, seed=3456, mode=None):
    w = b["w"]
    prec = Precision(mode or w.dtype)
    masters = b["masters"].copy()
    L, G = [], []
    for s in range(n_steps):
        l, g, masters = zo.zo_step(w, b["layout"], b["frozen"], masters, b["tokens"], b["labels"], seed, s, prec)
        L.append(l)
        G.append(g)
    return np.array(L), np.array(G), masters


def rel_err(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def oracle_traces(b, seed=3456, step=0, mode=None):
    """Per copy: residual stream after the embedding and after every block, and the loss.
    Returns (H[L+1][n*E*S, d] float32 stacked in copy-major order, losses[n])."""
    from oracle.model import copy_loss
    w = b["w"]
    prec = Precision(mode or w.dtype)
    traces, losses = [], []
    for k in range(w.q):
        z = zo.draw_z(b["layout"], seed, step, k, b["masters"].size, w.perturb_A)
        for sign in (+1, -1):
            theta = zo.perturb(b["masters"], z, sign, w.eps, prec)
            tr = []
            losses.append(copy_loss(w, b["frozen"], zo.split_factors(b["layout"], theta), b["tokens"], b["labels"],
                                    prec, trace=tr))
            traces.append(tr)
    L = len(traces[0])
    H = [np.concatenate([t[i].reshape(-1, w.d_model) for t in traces], axis=0).astype(np.float32) for i in range(L)]
    return H, np.array(losses)
