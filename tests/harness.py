"""Shared helpers of the GPU parity tests: drive the HIP library and the CPU oracle on the same seeded inputs."""
import numpy as np

import pp_inputs as gen
from oracle import pp_oracle as O

HP = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)


def cosine(a, b):
    a = np.asarray(a, dtype=np.float64).reshape(-1)
    b = np.asarray(b, dtype=np.float64).reshape(-1)
    na, nb = np.linalg.norm(a), np.linalg.norm(b)
    if na == 0 and nb == 0:
        return 1.0
    return float(a @ b / (na * nb + 1e-300))


def segment_slices(cfg, mask):
    """(name, packed offset, count) for every segment of the packed subset, in packed order."""
    out, off = [], 0
    d = cfg["d_model"]
    for name, lo, hi in O.mask_segments(cfg, mask):
        cnt = (hi - lo) * d
        out.append((f"{name}[{lo}:{hi}]", off, cnt))
        off += cnt
    return out


def expand_mask(cfg, mask):
    if mask.get("all"):
        return gen.all_mask(cfg)
    return mask


def make_gpu_model(cfg, weights, mask, force_plain=False):
    import paper_2509_22418_amd as pp
    m = pp.LocalStepModel(cfg, mask)
    m.load_weights(weights)
    if force_plain:
        m.set_option("force_plain", 1)
    m.set_mask()
    return m


def frozen_bytes_equal(cfg, model, weights_before, mask):
    """Every element outside I_train must be bit-identical to what was uploaded."""
    mask = expand_mask(cfg, mask)
    train = {}
    for name, lo, hi in O.mask_segments(cfg, mask):
        train.setdefault(name, []).append((lo, hi))
    bad = []
    for name, shape in gen.tensor_shapes(cfg).items():
        now = model.get_weight(name, shape)
        ref = np.asarray(weights_before[name], dtype=np.float32)
        keep = np.ones(shape[0] if len(shape) == 2 else 1, dtype=bool)
        for lo, hi in train.get(name, []):
            keep[lo:hi] = False
        a = now.reshape(keep.size, -1)[keep].view(np.uint32)
        b = ref.reshape(keep.size, -1)[keep].view(np.uint32)
        if not np.array_equal(a, b):
            bad.append(name)
    return bad
