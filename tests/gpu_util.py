"""Helpers for the GPU parity tests (host <-> device plumbing only)."""
import numpy as np
import torch

import gr_synth


def dev():
    return torch.device("cuda:0")


def bf16_to_dev(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev()).view(torch.bfloat16)


def bf16_to_host_f32(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy()


def to_dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(dev())


def run_attn(gr, a, scale, want_lse=True):
    B, W, Hq, d = a["q"].shape
    cu = a["cu_seqlens"]
    lse = torch.empty((B, W, Hq), dtype=torch.float32, device=dev()) if want_lse else None
    out, lse = gr.gr_beam_attn(bf16_to_dev(a["q"]), bf16_to_dev(a["k_shared"]), bf16_to_dev(a["v_shared"]), to_dev(cu),
                               bf16_to_dev(a["k_unshared"]), bf16_to_dev(a["v_unshared"]), a["u"], scale,
                               int(np.diff(cu).max()) if len(cu) > 1 else 0, int(cu[-1]), lse_out=lse)
    torch.cuda.synchronize()
    return bf16_to_host_f32(out), (lse.cpu().numpy() if lse is not None else None)


def rand_attn_case(seed, B, W, Hq, Hkv, d, ND, u, lens):
    rng = np.random.default_rng(seed)
    cu = np.zeros(B + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    total = max(int(cu[-1]), 1)
    bf = lambda *s: gr_synth.f32_to_bf16_bits(rng.standard_normal(s, dtype=np.float32))
    return dict(q=bf(B, W, Hq, d), k_shared=bf(total, Hkv, d), v_shared=bf(total, Hkv, d), cu_seqlens=cu,
                k_unshared=bf(B, W, ND, Hkv, d), v_unshared=bf(B, W, ND, Hkv, d), u=u)


def run_select(gr, mask, logits, sc, pf, rg, step, flags=0):
    r = gr.gr_beam_select(mask, to_dev(logits), to_dev(sc), to_dev(pf), to_dev(rg), step, flags=flags)
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in r.items()}


def assert_select_equal(got, want, msg=""):
    for k in ("parent", "token", "prefix", "range", "item_index"):
        np.testing.assert_array_equal(got[k], want[k], err_msg=f"{msg} {k}")
    fin = np.isfinite(want["scores"])
    np.testing.assert_array_equal(np.isfinite(got["scores"]), fin, err_msg=f"{msg} finite pattern")
    # spec bar: beam scores within 1e-5 relative (the canonical arithmetic makes them equal in practice)
    np.testing.assert_allclose(got["scores"][fin], want["scores"][fin], rtol=1e-5, atol=0, err_msg=f"{msg} scores")
    assert (got["scores"][~fin] == -np.inf).all()
