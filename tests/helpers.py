"""Shared test helpers: exact upcasts for the oracle and error metrics."""
import numpy as np
import torch


def f64(t):
    """Stored bits of a torch tensor, upcast exactly to a float64 numpy array."""
    return t.detach().cpu().double().numpy()


def max_abs(a, b):
    return float(np.max(np.abs(np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64)))) if np.size(a) else 0.0


def rmse(a, b):
    d = np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64)
    return float(np.sqrt(np.mean(d * d))) if d.size else 0.0


def rel_rmse(a, ref):
    ref = np.asarray(ref, dtype=np.float64)
    return rmse(a, ref) / max(float(np.sqrt(np.mean(ref * ref))), 1e-300)


def gpu_rows(t, rows):
    """Rows `rows` (flat over B*H*N) of a [B,H,N,d] or [B,H,N] device tensor, as float64 numpy."""
    idx = torch.from_numpy(rows).to(t.device)
    flat = t.reshape(-1, t.shape[-1]) if t.dim() == 4 else t.reshape(-1)
    return flat.index_select(0, idx).double().cpu().numpy()
