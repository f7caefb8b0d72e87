"""Helpers of the GPU parity tests: move seeded inputs to the GPU, run the oracle beside it."""
import numpy as np
import torch

from oracle import oracle as O
from paper_2602_11686_amd import binding as B
from paper_2602_11686_amd import inputs as I
from paper_2602_11686_amd.layer import MoeLayerBuffers, to_device

TOL = {torch.bfloat16: 2e-2, torch.float32: 1e-4}   # max|got-ref| / max|ref| per tensor


def tdtype(w):
    return torch.bfloat16 if w.dtype == "bf16" else torch.float32


def shape_of(w):
    return B.Shape(w.T, w.d, w.f, w.E, w.k, tdtype(w))


def host(t: torch.Tensor) -> np.ndarray:
    """GPU tensor -> numpy fp64 (floats) or its integer type."""
    t = t.detach().cpu()
    if t.dtype in (torch.bfloat16, torch.float32):
        return t.to(torch.float64).numpy()
    return t.numpy()


def round_like(a: np.ndarray, w) -> np.ndarray:
    """Oracle values rounded to the workload's storage type, as stored bits/values."""
    if w.dtype == "bf16":
        return I.f32_to_bf16_bits(a.astype(np.float32))
    return a.astype(np.float32)


def dev(a: np.ndarray, w):
    return to_device(a, tdtype(w))


def oracle_inputs(inp, real=np.float64):
    return {n: I.widen(v, real) for n, v in inp.items()}


def check_gate(ids_gpu, w_gpu, logits_gpu, ref_ids, ref_w, ref_logits, k):
    """Bit-exact ids wherever the oracle's margins exceed the accumulation noise; a token below the
    threshold is accepted iff the GPU's choice is a valid sorted top-k of the GPU's own logits.
    Returns the number of such near-tie tokens."""
    L = ref_logits
    live = L > -1e3                      # experts switched off by a -1e4 bias never compete
    scale = max(1.0, np.abs(L[live]).max())
    tau = 1e-5 * scale
    srt = -np.sort(-L, axis=1)
    gaps = np.abs(np.diff(srt[:, :min(k + 1, L.shape[1])], axis=1))
    safe = (gaps > tau).all(axis=1) if gaps.size else np.ones(L.shape[0], bool)
    np.testing.assert_array_equal(ids_gpu[safe], ref_ids[safe])
    if logits_gpu is not None:
        assert np.abs(logits_gpu - L)[live].max() <= 1e-5 * scale
        assert np.abs(logits_gpu - L).max() <= 1e-2      # fp32 spacing near the -1e4 bias is 1e-3
    for t in np.nonzero(~safe)[0]:
        assert logits_gpu is not None, "near-tie token needs the GPU's logits to be validated"
        lg = logits_gpu[t]
        order = np.argsort(-lg, kind="stable")[:k]
        np.testing.assert_array_equal(ids_gpu[t], order)
    same = (ids_gpu == ref_ids).all(axis=1)
    assert np.abs(w_gpu[same] - ref_w[same]).max() <= 2e-6 + 1e-5
    np.testing.assert_allclose(w_gpu.sum(1), 1.0, atol=1e-5)
    return int((~safe).sum())


def follow_gpu_ids(o, w, fw, ids_gpu):
    """The oracle's staged layer with the GPU's (validated) choice taken for the near-tie tokens.

    check_gate has accepted a token whose ids differ from the oracle's only if the gaps between the
    logits involved are below the accumulation noise and the GPU's ids are the sorted top-k of its own
    logits; downstream parity of such a token is defined on the ids the GPU returned.  The gate weights
    of those tokens are the softmax of the ORACLE's logits over the chosen experts.
    Returns (forward dict, backward dict or None, number of tokens that differ)."""
    from scipy.special import softmax
    differ = (ids_gpu != fw["ids"]).any(axis=1)
    if not differ.any():
        return fw, None, 0
    ids = np.where(differ[:, None], ids_gpu, fw["ids"]).astype(np.int32)
    tw = fw["w"].copy()
    sel = np.take_along_axis(fw["logits"][differ], ids_gpu[differ].astype(np.int64), axis=1)
    tw[differ] = softmax(sel, axis=1).astype(tw.dtype)
    counts, offsets, rop, por, Xp = O.permute(o["x"], ids, w.E)
    Yp, A, Bm, H = O.ffn_fwd(Xp, offsets, o["w1"], o["w3"], o["w2"])
    Y = O.unpermute_combine(Yp, rop, tw, w.T)
    fw2 = dict(ids=ids, w=tw, logits=fw["logits"], counts=counts, offsets=offsets, row_of_pair=rop,
               pair_of_row=por, Xp=Xp, Yp=Yp, A=A, B=Bm, H=H, Y=Y)
    bw2 = O.layer_bwd(o["x"], o["w_gate"], o["w1"], o["w3"], o["w2"], fw2, o["dy"]) if "dy" in o else None
    return fw2, bw2, int(differ.sum())
