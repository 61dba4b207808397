"""The two ceiling-measurement kernels run and do what prism.h says (tiny launches)."""
import pytest
import torch

import paper_2508_12851_amd as P

pytestmark = pytest.mark.gpu


def test_mfma_loop_counts_flop_and_computes_the_products():
    n_wg, iters = 4, 3
    ops = torch.full((n_wg * 256 * 16,), 0.5, dtype=torch.bfloat16, device="cuda")
    out = torch.empty(n_wg * 256, dtype=torch.float32, device="cuda")
    flop = P.prism_ceiling_mfma_bf16(ops, out, n_wg, iters)
    torch.cuda.synchronize()
    assert flop == n_wg * 4 * iters * 8 * 2 * 32 * 32 * 16
    # every accumulator element is iters * 16 * 0.25; a thread sums its 8 * 16 elements
    assert torch.all(out == iters * 16 * 0.25 * 8 * 16)


def test_stream_read_touches_the_whole_buffer():
    src = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    src[-16:] = 0x5A                       # last 16-byte vector must be seen by some thread
    sink = torch.zeros(8 * 256 * 16, dtype=torch.uint8, device="cuda")
    assert P.prism_ceiling_hbm_read(src, sink, 8) == 1 << 20
    torch.cuda.synchronize()
    assert int((sink == 0x5A).sum()) == 16


def test_ceiling_calls_reject_bad_arguments():
    ops = torch.zeros(4 * 256 * 16, dtype=torch.bfloat16, device="cuda")
    out = torch.empty(4 * 256, dtype=torch.float32, device="cuda")
    with pytest.raises(P.PrismError):
        P.prism_ceiling_mfma_bf16(ops, out, 0, 3)
    with pytest.raises(P.PrismError):
        P.prism_ceiling_hbm_read(ops[1:], out, 4)      # misaligned source


@pytest.mark.parametrize("mode", [0, 1, 2, 3])
@pytest.mark.parametrize("u", [2, 16])
def test_patterned_stream_read_touches_every_span(mode, u):
    """Each access pattern reads every 16-byte vector of the spans it reports: a marker in the
    last vector of the last span is seen (modes 0 and 2 hand the data to a register, whose xor is
    stored; the direct-to-LDS modes leave it in LDS, where one lane picks it up)."""
    span = 4096 * u
    n_spans = 5
    src = torch.zeros(span * n_spans + 100, dtype=torch.uint8, device="cuda")    # a ragged tail is not read
    src[span * n_spans - 16: span * n_spans] = 0x3C
    sink = torch.zeros(8 * 4096, dtype=torch.uint8, device="cuda")
    assert P.prism_ceiling_hbm_read_pattern(src, sink, 3, u, span, mode) == span * n_spans
    torch.cuda.synchronize()
    assert int((sink == 0x3C).sum()) == 16


def test_patterned_stream_read_rejects_what_the_header_rules_out():
    src = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(8 * 4096, dtype=torch.uint8, device="cuda")
    for kw in (dict(loads_in_flight=3, span_bytes=16384, mode=0), dict(loads_in_flight=4, span_bytes=1000, mode=0),
               dict(loads_in_flight=4, span_bytes=16384, mode=7), dict(loads_in_flight=4, span_bytes=2 << 20, mode=0)):
        with pytest.raises(P.PrismError):
            P.prism_ceiling_hbm_read_pattern(src, sink, 4, **kw)
