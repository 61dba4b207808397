"""Which error measure the random-shape GPU parity cases are held to, settled on the CPU.

The output bar is max |a - ref| / (|ref| + rms(ref)) <= 2e-2 for bf16, the rms taken over the
whole batch.  For a layer whose tokens differ by orders of magnitude in size, the roundings
the bf16 layer is defined with (silu*up, every expert output row and the sum each stored as
bf16) can exceed that bar in otherwise exact arithmetic; no kernel could then pass, and such a
case is held to the same formula with the rms of the token's own row.  This test runs the
rounding-point emulation (tests/rounding_emulation.py) on every random case and shows that the
cases listed in random_cases.PER_ROW_CASES are exactly those, and that every stage of every
other case stays under the whole-batch bar with room for the kernels' fp32 accumulation."""
import numpy as np
import pytest

from oracle import prism_oracle as O
from prism_inputs import make_config, make_inputs
from random_cases import N_CASES, PER_ROW_CASES, draw_case
from rounding_emulation import emulate

TOL_BF16 = 2e-2


def _err(a, ref, per_row=False):
    a, ref = np.asarray(a, np.float64), np.asarray(ref, np.float64)
    if ref.size == 0:
        return 0.0
    rms = np.sqrt(np.mean(ref ** 2, axis=-1, keepdims=True)) if per_row else np.sqrt(np.mean(ref ** 2))
    diff = np.abs(a - ref)
    return float(np.max(np.where(diff == 0, 0.0, diff / (np.abs(ref) + rms + 1e-300))))


@pytest.fixture(scope="module")
def table():
    rows = {}
    for i in range(min(N_CASES, 32)):
        kw, gate_mode, _ = draw_case(i)
        cfg = make_config("cfg4_finegrained", **kw)
        inp = make_inputs(cfg)
        f = inp.f32
        experts = lambda e: tuple(f(w) for w in inp.expert(e))
        shared = [tuple(f(w) for w in inp.shared(s)) for s in range(cfg.S)]
        ref = O.moe_layer(f(inp.x), f(inp.w_router), inp.bias, experts, shared, inp.mask, cfg.k,
                          cfg.dtype, cfg.bias_group_tokens, None, gate_mode == "renormalized")
        d = ref.dispatch
        refs = dict(out=ref.out,
                    y=O.expert_ffn(f(inp.x), experts, shared, d.local_src, d.local_offsets, cfg.k),
                    y_remote=O.expert_ffn(f(inp.x), experts, [], d.remote_src, d.remote_offsets, cfg.k))
        refs["done"] = O.combine_remote(ref.out, refs["y_remote"], d.remote_src, ref.route.topk_gate,
                                        cfg.dtype)
        em = emulate(inp, ref.route, d)
        rows[i] = (cfg.dtype, {n: (_err(em[n], refs[n]), _err(em[n], refs[n], True)) for n in refs})
    return rows


def test_only_the_listed_cases_exceed_the_whole_batch_bar_in_exact_arithmetic(table):
    over = {i for i, (dtype, e) in table.items() if dtype == "bf16" and e["out"][0] > TOL_BF16}
    assert over == set(PER_ROW_CASES) & set(table), over
    for i in over:
        whole, per_row = table[i][1]["out"]
        print(f"case {i}: roundings alone give {whole:.4f} against the batch rms, {per_row:.4f} against the row rms")
        assert per_row <= 0.6 * TOL_BF16


def test_every_other_stage_and_case_has_room_under_the_whole_batch_bar(table):
    for i, (dtype, e) in table.items():
        for name, (whole, _) in e.items():
            if i in PER_ROW_CASES and name == "out":
                continue
            bar = 1.5 * TOL_BF16 if name == "done" else TOL_BF16     # one more rounding on the way
            assert whole <= 0.9 * bar, (i, name, whole)
            if dtype == "f32":
                assert whole <= 1e-6, (i, name, whole)                # fp32 storage: no visible rounding


def test_case_12_figure(table):
    """The figure the GPU kernels show for this case under the whole-batch measure (0.0235) is
    the roundings' own: the emulation gives the same to three digits."""
    if 12 in table:
        assert abs(table[12][1]["out"][0] - 0.0235) < 5e-4
