"""Shared plumbing of the GPU parity tests: dtype conversion between the seeded fp32 inputs,
the fp64 oracle and device tensors, and the error metric of the parity bar."""
import numpy as np
import torch

import synth_inputs as synth

TOL = {"bf16": 2e-2, "f32": 1e-4}
TORCH_DT = {"bf16": torch.bfloat16, "f32": torch.float32}


def to_dev(x, dtype):
    """fp32 numpy (already rounded to `dtype`) -> device tensor of that dtype, same values."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    return t.to(TORCH_DT[dtype]).cuda()


def to_np(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def f64(d):
    return {k: np.asarray(v, dtype=np.float64) for k, v in d.items()}


def rel_err(gpu, ref):
    ref = np.asarray(ref, dtype=np.float64)
    scale = np.abs(ref).max()
    if scale == 0:
        return float(np.abs(gpu).max())
    return float(np.abs(gpu - ref).max() / scale)


def cosine(gpu, ref):
    a, b = np.asarray(gpu).ravel(), np.asarray(ref).ravel()
    n = np.linalg.norm(a) * np.linalg.norm(b)
    return float(a @ b / n) if n > 0 else 1.0


def check_all(out, ref, tol, label, keys=None, min_cosine=0.999):
    """Parity bar on every output tensor: max|gpu - oracle| / max|oracle| <= tol.  The cosine similarity is
    reported beside it (printed with -s / on failure) and must not fall below min_cosine."""
    rows, worst = [], 0.0
    for k in (keys if keys is not None else out.keys()):
        g = to_np(out[k])
        e, c = rel_err(g, ref[k]), cosine(g, ref[k])
        rows.append("%s %-8s rel_err %.3e  cosine %.6f" % (label, k, e, c))
        worst = max(worst, e)
    print("\n".join(rows), flush=True)
    for k, line in zip((keys if keys is not None else out.keys()), rows):
        g = to_np(out[k])
        assert rel_err(g, ref[k]) <= tol, line
        assert cosine(g, ref[k]) >= min_cosine, line
    return worst


def oracle_shape(shp):
    from oracle import LayerShape
    return LayerShape(shp["hidden"], shp["n_q_heads"], shp["n_kv_heads"], shp["head_dim"], shp["ffn"],
                      shp["rms_eps"], shp["rope_base"])


def alch_shape(shp, dtype):
    import paper_2503_01066_amd as A
    return A.make_shape(shp["hidden"], shp["n_q_heads"], shp["n_kv_heads"], shp["head_dim"], shp["ffn"],
                        shp["rms_eps"], shp["rope_base"], dtype)
