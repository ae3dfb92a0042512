"""The decoder-stack loop: every fused linear inside it against the oracle on the inputs it actually
saw, and HIP-graph replays against the eager pass."""
import numpy as np
import pytest

import fbq_synth
from helpers import assert_matches_oracle, make_oracle_layer, oracle_y, to_device_layer

pytestmark = pytest.mark.gpu

Y_TOL = 1e-3          # relative L2 per linear layer, as for the single-layer tests
HIDDEN, INTER, RANK = 256, 640, 16


@pytest.mark.parametrize("batch", [1, 5, 72])      # one row (GEMV), a few (matrix-core decode), a prompt pass (prefill GEMM)
@pytest.mark.parametrize("bits", [4, 3])
def test_decoder_stack_linears_match_oracle_and_graph_replays_are_exact(bits, batch):
    import torch
    from paper_2501_16385_amd.decode_loop import DecoderStack, NAMES, layer_shapes

    shapes = layer_shapes(HIDDEN, INTER)
    oracle_layers, dev_layers = [], []
    for li in range(2):
        ol = {}
        for j, n in enumerate(NAMES):
            spec = fbq_synth.LayerSpec(n, shapes[n][0], shapes[n][1], RANK, bits)
            ol[n] = make_oracle_layer(spec, config=40 + bits, layer_index=7 * li + j)
        oracle_layers.append(ol)
        dev_layers.append({n: to_device_layer(ol[n]) for n in NAMES})

    x0 = fbq_synth.make_x(fbq_synth.LayerSpec("x", HIDDEN, HIDDEN, 0, bits), batch, 40 + bits, 0)
    x0d = torch.from_numpy(x0.view(np.int16)).cuda().view(torch.float16)

    stack = DecoderStack(dev_layers, HIDDEN, INTER, keep_per_layer_buffers=True, batch=batch)
    stack.x.copy_(x0d)
    stack.step()
    torch.cuda.synchronize()
    eager = stack.x.cpu().numpy().copy()
    assert np.all(np.isfinite(eager))

    # every linear on the input it saw (x_in, v, h, act) against the oracle
    host = lambda t: t.cpu().numpy()
    for li in range(2):
        b = stack.buf[li]
        inputs = {"q": b["x_in"], "k": b["x_in"], "v": b["x_in"], "o": b["v"], "gate": b["h"], "up": b["h"], "down": b["act"]}
        for n in NAMES:
            want = oracle_y(oracle_layers[li][n], host(inputs[n]))
            assert_matches_oracle(host(b[n]), want, f"layer {li} {n}", tol=Y_TOL)

    # graph replays, with eager work and synchronisation between them, reproduce the eager pass bit for bit
    graph = stack.capture()
    for rep in range(3):
        stack.x.copy_(x0d)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(stack.x.cpu().numpy(), eager), f"replay {rep} differs from the eager pass"
        (stack.buf[0]["q"] * 2).sum().item()      # unrelated eager work between replays
