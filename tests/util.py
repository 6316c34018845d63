"""Helpers shared by the GPU parity tests: build the device scene and the oracle scene from the
same seeded arrays."""
import numpy as np

import kn_synth as ks
from oracle import OracleScene

TORCH_DTYPE = {"f32": "float32", "f16": "float16", "bf16": "bfloat16"}


def device_weights(w_rounded_f32, wdtype):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(w_rounded_f32))
    return t.to(getattr(torch, TORCH_DTYPE[wdtype])).cuda().contiguous()   # exact: values are representable


def make_pair(sc, threads=False):
    """sc: scene dict from kn_synth.configs -> (device Scene, OracleScene)."""
    import torch
    import paper_2103_13744_amd as kn
    occ = sc["occupancy"]
    table = sc.get("cell_net")          # sparse network grid: cell -> row of weights, or None
    dev = kn.Scene(sc["res"], sc["aabb_min"], sc["aabb_max"], sc["hidden"], device_weights(sc["weights"], sc["wdtype"]),
                   None if occ is None else torch.from_numpy(occ).cuda(),
                   cell_net=None if table is None else torch.from_numpy(table).cuda())
    orc = OracleScene(sc["res"], sc["aabb_min"], sc["aabb_max"], sc["hidden"], sc["weights"], occ, threads=threads,
                      cell_net=table)
    return dev, orc


def scene_dict(res, lo, hi, hidden, wdtype, seed, occ=None, sigma_scale=1.0):
    n = int(np.prod(res))
    w = ks.round_to_storage(ks.kaiming_weights(n, hidden, seed, sigma_scale=sigma_scale), wdtype)
    return dict(res=tuple(res), aabb_min=tuple(lo), aabb_max=tuple(hi), hidden=hidden, wdtype=wdtype, weights=w,
                occupancy=occ, L_pos=10, L_dir=4)


def cuda(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()
