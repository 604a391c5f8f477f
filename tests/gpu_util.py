"""Helpers shared by the GPU parity tests (marshalling only)."""
import os

import numpy as np
import torch

from oracle import dit

from paper_2509_06040_amd import binding as br
from paper_2509_06040_amd import synth

DEV = "cuda"


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    return t.to(dtype) if dtype is not None else t


def host(t):
    torch.cuda.synchronize()
    return t.detach().float().cpu().numpy() if t.dtype == torch.bfloat16 else t.detach().cpu().numpy()


def bytes_buffer(n):
    return torch.empty(max(int(n), 256), dtype=torch.uint8, device=DEV)


def rel_l2(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def make_model(cfg, W):
    return br.Model(cfg, br.upload_weights(cfg, W))


def cond_dev(cfg, cond):
    return dev(cond, torch.bfloat16 if cfg["dtype"] == synth.BF16 else torch.float32)


def velocity_errors(cfg, got, ref):
    """Error measures of one sample's velocity against the oracle's: (relative L2 over the sample,
    worst relative L2 over the image tokens -- a token's reference norm is floored at half the
    sample's RMS token norm --, largest element error in units of the sample's RMS)."""
    g = dit.patchify(cfg, np.asarray(got, np.float64)[None])[0]
    r = dit.patchify(cfg, np.asarray(ref, np.float64)[None])[0]
    err_tok = np.linalg.norm(g - r, axis=1)
    ref_tok = np.linalg.norm(r, axis=1)
    floor = 0.5 * np.sqrt((ref_tok ** 2).mean())
    rms = np.sqrt((r ** 2).mean())
    return (float(np.linalg.norm(g - r) / max(np.linalg.norm(r), 1e-300)),
            float((err_tok / np.maximum(ref_tok, floor)).max()),
            float(np.abs(g - r).max() / max(rms, 1e-300)))


def assert_velocity(cfg, got, ref, tol, what=""):
    """Teacher-forced velocity check at tolerance `tol` (1e-4 fp32, 2e-2 bf16): the whole sample and
    every single token within `tol` in relative L2, every element within 4 tol of the sample's RMS.
    One wrong token, or one wrong element, fails even where the sample norm would hide it."""
    rel, tok, mx = velocity_errors(cfg, got, ref)
    if os.environ.get("BR_TEST_VERBOSE"):
        print("velocity %s: rel %.3e, worst token %.3e, max element %.3e rms" % (what, rel, tok, mx), flush=True)
    assert rel <= tol, (what, "sample", rel)
    assert tok <= tol, (what, "token", tok)
    assert mx <= 4 * tol, (what, "element", mx)


def assert_tokens(got, ref, tol, what=""):
    """The same bar on a subset of a sample's tokens (rows = tokens): all rows together and every
    single row within `tol` in relative L2 (row norms floored at half their RMS), every element
    within 4 tol of the rows' RMS."""
    g, r = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    err_tok, ref_tok = np.linalg.norm(g - r, axis=1), np.linalg.norm(r, axis=1)
    floor = 0.5 * np.sqrt((ref_tok ** 2).mean())
    rel = float(np.linalg.norm(g - r) / max(np.linalg.norm(r), 1e-300))
    tok = float((err_tok / np.maximum(ref_tok, floor)).max())
    mx = float(np.abs(g - r).max() / max(np.sqrt((r ** 2).mean()), 1e-300))
    if os.environ.get("BR_TEST_VERBOSE"):
        print("tokens %s: rel %.3e, worst token %.3e, max element %.3e rms" % (what, rel, tok, mx), flush=True)
    assert rel <= tol, (what, "rows", rel)
    assert tok <= tol, (what, "token", tok)
    assert mx <= 4 * tol, (what, "element", mx)
