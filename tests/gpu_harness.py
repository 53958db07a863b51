"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI,
run the oracle on the same bytes, compare field by field.

Parity bar: medians, MADs, masks, anomaly bits, counters, flags, first-flag
steps and top-k (indices and keys) bit-exact; node scores bit-exact; z within
1e-6 relative (in practice bit-exact as well, which is reported).  Comparisons
whose score lies within 1e-5 (relative) of the threshold are counted by the
oracle and reported separately.
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2605_17879_amd import Config, Detector

Z_RTOL = 1e-6
# None: the library's own choice between one workgroup per run of steps and one per
# column; 0: never per column; 64: per column whenever the columns fit the chip.
STREAMING_STEPS = None


def oracle_params(w=None, **kw) -> oracle.Params:
    if w is not None:
        base = dict(R=w.R, M=w.M, W=w.W, k=w.k, thr=w.thr, directions=tuple(w.directions),
                    primary=w.primary, min_signals=w.min_signals)
        base.update(kw)
        kw = base
    return oracle.Params(**kw)


def detector_for(p: oracle.Params, topk=None) -> Detector:
    cfg = Config(n_ranks=p.R, n_metrics=p.M, window=p.W, persist_k=p.k, gpus_per_node=p.G,
                 primary_metric=p.primary, min_signals=p.min_signals, topk=topk,
                 node_agg=p.node_agg, z_threshold=p.thr, node_scale=p.node_scale,
                 rel_floor=p.rel_floor, abs_floor=p.abs_floor,
                 direction=tuple(p.directions)[: p.M])
    det = Detector(cfg)
    if STREAMING_STEPS is not None:
        det.set_streaming_steps(STREAMING_STEPS)
    return det


def u64(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint64)


def gpu_score(det: Detector, x: torch.Tensor, want_z=True) -> dict:
    xd = x.cuda() if not x.is_cuda else x
    out = det.alloc_outputs(xd.shape[0], want_z=want_z)
    # poison the outputs so that an element the kernel forgets to write shows up
    for k, v in out.items():
        if v is not None:
            v.view(torch.uint8).fill_(0xA5)
    det.score_batch(xd, out)
    torch.cuda.synchronize()
    return out


def bits32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def compare_scores(o: oracle.Scores, g: dict, label="") -> dict:
    """Assert parity of one gd_score_batch call; returns a small report."""
    rep = {}
    med, mad = g["med"].cpu().numpy(), g["mad"].cpu().numpy()
    assert np.array_equal(bits32(med), bits32(o.med)), f"{label}: medians differ"
    assert np.array_equal(bits32(mad), bits32(o.mad)), f"{label}: MADs differ"
    assert np.array_equal(g["exceed_mask"].cpu().numpy(), o.exceed_mask), f"{label}: exceed masks differ"
    assert np.array_equal(u64(g["rank_anom"]), o.rank_anom), f"{label}: rank anomaly bits differ"
    assert np.array_equal(bits32(g["node_z"].cpu().numpy()), bits32(o.node_z)), f"{label}: node scores differ"
    assert np.array_equal(g["node_mask"].cpu().numpy(), o.node_mask), f"{label}: node masks differ"
    assert np.array_equal(u64(g["node_anom"]), o.node_anom), f"{label}: node anomaly bits differ"
    if g.get("z") is not None and o.z is not None:
        z = g["z"].cpu().numpy()
        err = np.abs(z.astype(np.float64) - o.z.astype(np.float64))
        tol = Z_RTOL * np.abs(o.z.astype(np.float64))
        assert np.all(err <= tol), f"{label}: z beyond {Z_RTOL} relative (max err {err.max()})"
        rep["z_bit_exact"] = bool(np.array_equal(bits32(z), bits32(o.z)))
    rep["near_rank"], rep["near_node"] = o.near_rank, o.near_node
    return rep


def gpu_flags(det: Detector) -> dict:
    f = det.alloc_flags()
    for v in f.values():
        v.view(torch.uint8).fill_(0xA5)
    det.flags(f)
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in f.items()}


def gpu_topk(det: Detector, k: int):
    tk = det.alloc_topk(k)
    det.topk_nodes(k, tk)
    torch.cuda.synchronize()
    return tk["idx"].cpu().numpy(), tk["key"].cpu().numpy().view(np.uint64)


def compare_severity(p: oracle.Params, d: dict, det: Detector, x: torch.Tensor, out: dict,
                     moderate=0.10, severe=0.20, label="") -> dict:
    """gd_severity on the batch x (scored into `out`, window already updated) against the
    oracle's tiers computed from ITS medians and flags (d = oracle.detect of the same history)."""
    xd = x.cuda() if not x.is_cuda else x
    sev = det.alloc_severity()
    for v in sev.values():
        v.view(torch.uint8).fill_(0xA5)
    det.severity(xd, out, sev, moderate, severe)
    torch.cuda.synchronize()
    T = x.shape[0]
    med = d["scores"].med[-T:] if T else d["scores"].med[:0]
    want_slow, want_tier = oracle.severity(p, x.cpu().numpy(), med, d["node_flag_byte"], moderate, severe)
    slow, tier = sev["slowdown"].cpu().numpy(), sev["tier"].cpu().numpy()
    assert np.array_equal(tier, want_tier), f"{label}: tiers differ"
    assert np.array_equal(bits32(slow), bits32(want_slow)), f"{label}: slowdowns differ"
    return {"tiers": np.bincount(want_tier, minlength=4).tolist()}


def compare_decision(p: oracle.Params, d: dict, det: Detector, topk_k: int, label=""):
    """d = oracle.detect(...) over the whole history the detector has consumed."""
    f = gpu_flags(det)
    assert np.array_equal(f["rank_count"].view(np.uint16), d["ranks"].count), f"{label}: rank counts"
    assert np.array_equal(f["rank_flag"], d["ranks"].flag), f"{label}: rank flags"
    assert np.array_equal(f["rank_first"], d["ranks"].first), f"{label}: rank first-flag steps"
    assert np.array_equal(f["node_count"].view(np.uint16), d["nodes"].count), f"{label}: node counts"
    assert np.array_equal(f["node_flag"], d["node_flag_byte"]), f"{label}: node flag bytes"
    assert np.array_equal(f["node_first"], d["nodes"].first), f"{label}: node first-flag steps"
    idx, key = gpu_topk(det, topk_k)
    assert np.array_equal(idx, d["topk_idx"]), f"{label}: top-k indices"
    assert np.array_equal(key, d["topk_key"]), f"{label}: top-k keys"


def run_and_compare(p: oracle.Params, x: torch.Tensor, topk_k: int, chunks=None, label="",
                    want_z=True) -> dict:
    """Whole path on x[T][M][R] (CPU tensor): oracle vs HIP, fed in `chunks` pieces."""
    T = x.shape[0]
    xn = x.numpy()
    d = oracle.detect(p, xn, topk_k=topk_k, want_z=want_z)
    det = detector_for(p)
    chunks = chunks or [T]
    assert sum(chunks) == T
    t0 = 0
    rep = {"z_bit_exact": True}
    for c in chunks:
        if c == 0:
            continue
        g = gpu_score(det, x[t0:t0 + c], want_z=want_z)
        o = d["scores"]
        part = oracle.Scores(o.med[t0:t0 + c], o.mad[t0:t0 + c],
                             None if o.z is None else o.z[t0:t0 + c],
                             o.exceed_mask[t0:t0 + c], o.rank_anom[t0:t0 + c], o.node_z[t0:t0 + c],
                             o.node_mask[t0:t0 + c], o.node_anom[t0:t0 + c], None, 0, 0)
        r = compare_scores(part, g, label=f"{label}[{t0}:{t0 + c}]")
        rep["z_bit_exact"] &= r.get("z_bit_exact", True)
        det.update_window(g, c)
        t0 += c
    compare_decision(p, d, det, topk_k, label=label)
    rep["near_rank"], rep["near_node"] = d["scores"].near_rank, d["scores"].near_node
    rep["rank_flags"] = int(d["ranks"].flag.sum())
    rep["node_flags"] = int((d["node_flag_byte"] & 1).sum())
    det.close()
    return rep
