"""Helpers for the GPU parity tests: move stored 16-bit patterns between numpy and device
buffers, build the device-side layer from an oracle-side case, and check a layer trace
stage by stage (teacher-forced: the oracle is applied to the GPU's own stage inputs)."""
from __future__ import annotations

import numpy as np
import torch

from oracle import larosa_oracle as O

REL_L2_TOL = 2e-3          # fp16/bf16 outputs with fp32 accumulation (target stated for this path)


def to_dev(bits: np.ndarray, dtype: str, device="cuda:0") -> torch.Tensor:
    if bits is None:
        return None
    td = torch.float16 if dtype == "f16" else torch.bfloat16
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(td)


def to_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def rel_l2(got: np.ndarray, want: np.ndarray) -> float:
    den = np.linalg.norm(want)
    return float(np.linalg.norm(got - want) / den) if den > 0 else float(np.linalg.norm(got))


ULP_FRACTION = 0.02       # share of entries that may sit one unit in the last place off the oracle's rounding


def _ordered(bits: np.ndarray) -> np.ndarray:
    """16-bit patterns as integers that count representable values (sign-magnitude -> two's complement)."""
    b = bits.astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7FFF), b)


def stored_close(got_bits: np.ndarray, want64: np.ndarray, dtype: str, what: str, tol=REL_L2_TOL) -> float:
    """A stored 16-bit tensor against the oracle's value after the same single rounding: relative L2 within
    `tol`, AND entry by entry at most one unit in the last place away, on at most ULP_FRACTION of the entries.
    Entries whose absolute error is below 2^-16 of the tensor's rms are accepted whatever their ulp count: the
    fp32 accumulation of a few thousand products is that uncertain, and for an entry that nearly cancels it is
    more than the entry's own (tiny) ulp.  Returns the relative L2 error."""
    want_bits = O.encode16(want64, dtype)
    got, want = O.decode16(got_bits, dtype), O.decode16(want_bits, dtype)
    e = rel_l2(got, want)
    assert e <= tol, f"{what}: rel-L2 {e:.3e} > {tol:.1e}"
    step = np.abs(_ordered(np.asarray(got_bits)) - _ordered(want_bits))
    err = np.abs(got - want)
    floor = 2.0 ** -16 * float(np.sqrt(np.mean(want * want))) if want.size else 0.0
    bad = (step > 1) & (err > floor)
    assert not bad.any(), (f"{what}: {int(bad.sum())} of {bad.size} entries beyond 1 ulp, worst {int(step[bad].max())} ulp, "
                           f"abs err {err[bad].max():.3e} (floor {floor:.3e})")
    frac = float(((step != 0) & (err > floor)).mean()) if step.size else 0.0
    assert frac <= ULP_FRACTION, f"{what}: {frac:.4f} of the entries are one ulp off"
    return e


def device_layer(case, device="cuda:0"):
    from paper_2507_01299_amd import api
    L, b, dt = case.layer, case.bits, case.shape.dtype
    return api.Layer(L.d, L.d_q, L.d_kv, L.d_ff, L.head_dim, L.K1, L.K2, L.K3, L.K4,
                     Wqkv=to_dev(b["Wqkv"], dt, device), Wo=to_dev(b["Wo"], dt, device),
                     Wgu=to_dev(b["Wgu"], dt, device), Wdown=to_dev(b["Wdown"], dt, device), dtype=dt,
                     Q_attn=to_dev(b.get("Q_attn"), dt, device), Q_mlp=to_dev(b.get("Q_mlp"), dt, device),
                     adapter=to_dev(b.get("adapter"), dt, device), rms_attn=to_dev(b.get("rms_attn"), dt, device),
                     rms_mlp=to_dev(b.get("rms_mlp"), dt, device), rms_eps=L.rms_eps,
                     shortcut_attn=to_dev(b.get("shortcut_attn"), dt, device),
                     shortcut_mlp=to_dev(b.get("shortcut_mlp"), dt, device))


def check_layer_trace(L: O.Layer, x_bits: np.ndarray, trace: dict, x_out: torch.Tensor, tol=REL_L2_TOL,
                      attn_bits: np.ndarray | None = None) -> dict:
    """Every stage of the GPU trace against the oracle applied to the GPU's own inputs of that
    stage.  Index arrays must be equal; 16-bit tensors within tol relative L2 and, entry by entry, within
    one unit in the last place on a bounded share of the entries (stored_close).  Returns the
    worst relative error per stage.  attn_bits: the output of a caller's attention core that was
    handed to the second half of a split layer run; h2 must then be exactly that."""
    dt = L.dtype
    g = {k: (v.cpu().numpy() if k.startswith("idx") else to_bits(v)) for k, v in trace.items() if v is not None}
    g["x_out"] = to_bits(x_out)
    B = x_bits.shape[0]
    worst = {}

    def close(name, got_bits, want64):
        e = stored_close(got_bits, want64, dt, name, tol)
        worst[name] = max(worst.get(name, 0.0), e)

    for b in range(B):
        x = O.decode16(x_bits[b], dt)
        close("h1", g["h1"][b], O.block_input(x, L.Q_attn, L.rms_attn, L.rms_eps, dt))
        assert np.array_equal(g["idx1"][b], O.topk_indices(g["h1"][b], L.K1)), "idx1"
        h1 = O.decode16(g["h1"][b], dt)
        close("qkv", g["qkv"][b], O.stage_qkv(L, h1, g["idx1"][b], dt))
        qkv = O.decode16(g["qkv"][b], dt)
        want_h2 = (attn_bits[b] if attn_bits is not None
                   else O.encode16(O.gqa_single_key_attention(qkv, L.d_q, L.d_kv, L.head_dim), dt))
        assert np.array_equal(g["h2"][b], want_h2), "h2"
        assert np.array_equal(g["idx2"][b], O.topk_indices(g["h2"][b], L.K2)), "idx2"
        h2 = O.decode16(g["h2"][b], dt)
        o, x1 = O.stage_attn_out(L, x, h2, g["idx2"][b], dt)
        close("o", g["o"][b], o)
        s1 = x
        if L.shortcut_attn is not None:
            close("s1", g["s1"][b], O.stage_shortcut(x, L.shortcut_attn, dt))
            s1 = O.decode16(g["s1"][b], dt)
        # the residual add is checked from the GPU's own o (and shortcut value)
        close("x1", g["x1"][b], O.round16(s1 + O.decode16(g["o"][b], dt), dt))
        x1g = O.decode16(g["x1"][b], dt)
        close("h3", g["h3"][b], O.block_input(x1g, L.Q_mlp, L.rms_mlp, L.rms_eps, dt))
        assert np.array_equal(g["idx3"][b], O.topk_indices(g["h3"][b], L.K3)), "idx3"
        h3 = O.decode16(g["h3"][b], dt)
        close("gu", g["gu"][b], O.stage_gate_up(L, h3, g["idx3"][b], dt))
        gu = O.decode16(g["gu"][b], dt)
        close("h4", g["h4"][b], O.stage_h4(L, gu, dt))
        assert np.array_equal(g["idx4"][b], O.topk_indices(g["h4"][b], L.K4)), "idx4"
        h4 = O.decode16(g["h4"][b], dt)
        dn, _ = O.stage_down(L, x1g, h4, g["idx4"][b], dt)
        close("down", g["down"][b], dn)
        s2 = x1g
        if L.shortcut_mlp is not None:
            close("s2", g["s2"][b], O.stage_shortcut(x1g, L.shortcut_mlp, dt))
            s2 = O.decode16(g["s2"][b], dt)
        x2_want = O.round16(s2 + O.decode16(g["down"][b], dt), dt)
        if L.adapter is not None:
            close("x2", g["x2"][b], x2_want)
            close("x_out", g["x_out"][b], O.stage_adapter(L, O.decode16(g["x2"][b], dt), dt))
        else:
            close("x_out", g["x_out"][b], x2_want)
    return worst


def free_run_index_disagreement(L: O.Layer, x_bits: np.ndarray, trace: dict) -> dict:
    """Informational: how many kept indices differ between the GPU run and a free-running
    oracle layer (differences arise only at near-ties after a one-ulp storage difference)."""
    out = {}
    for b in range(x_bits.shape[0]):
        r = O.layer_forward(L, O.decode16(x_bits[b], L.dtype), rounded=True)
        for k in ("idx1", "idx2", "idx3", "idx4"):
            gi = set(trace[k][b].cpu().numpy().tolist())
            out[k] = out.get(k, 0) + len(gi.symmetric_difference(set(r[k].tolist()))) // 2
    return out
