"""Oracle scores of whole layers in worker processes (numpy only: the workers never touch the GPU and
do not import torch), for GPU tests that compare every unit of a large configuration."""
from __future__ import annotations

import multiprocessing as mp
import os

os.environ.setdefault("OMP_NUM_THREADS", "1")

import numpy as np

from oracle import mixkv_oracle as O
from paper_2510_20707_amd import synth


def _layer_scores(job):
    name, over, layer_id, params = job
    wl = synth.WORKLOADS[name].with_(**over) if over else synth.WORKLOADS[name]
    lay = synth.make_layer(wl, layer_id)
    p = O.Params(**params)
    G = wl.group
    out = {}
    for b in range(wl.batch):
        for h in range(wl.n_kv_heads):
            u = O.score_unit(lay.K[b, h], lay.V[b, h], lay.Q[b, h * G:(h + 1) * G], p)
            out[(b, h)] = dict(s_comp=u["s_comp"], r=float(u["r"]))
    return layer_id, out


def score_layers(name: str, over: dict, layer_ids, params: dict, workers: int = 8):
    """{layer_id: {(b, h): {"s_comp", "r"}}} for the given layers of workload `name` (with_ overrides
    `over`), `params` being the keyword arguments of oracle.Params.  Spawned workers: the caller may
    have initialised the GPU, which a forked child must not inherit."""
    jobs = [(name, over, l, params) for l in layer_ids]
    ctx = mp.get_context("spawn")
    with ctx.Pool(min(workers, len(jobs))) as pool:
        return dict(pool.map_async(_layer_scores, jobs, chunksize=1).get(timeout=900))
