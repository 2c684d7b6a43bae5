"""bnn_forward_static (the forward pass for callers that cannot allocate: its ping-pong buffers are a fixed array in the
library's device image) against bnn_forward with a caller workspace: the same kernels on the same inputs, so every
output bit is the same.  Two calls in a row, the second on a smaller batch, so that what the first call left in the
array is seen not to matter."""
import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def test_forward_static_matches_forward_on_two_calls_in_a_row():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import harness as G
    import paper_1706_09453_amd as bnn

    for cid, batches in ((3, (1500, 333)), (8, (1100, 70)), (10, (300, 96))):
        cfg = workloads.CONFIGS[cid]
        Ws, bs = workloads.make_net_params(cfg)
        model = G.GpuModel(Ws, bs, cfg.hidden_act, cfg.word_bits, real_weight_layers=cfg.real_weight_layers)
        for M in batches:
            X = G.to_dev(workloads.make_frames(cfg, M))
            # Config 10 at 300 frames: the bf16 planes of its Softmax layer (six bytes per weight) do not fit the fixed
            # array, so the static entry point runs that layer on the fp32 matrix cores, as bnn_forward does with the
            # option off
            fits = bnn.bnn_forward_workspace_bytes(model.layers, model.n_layers, M) <= bnn.BNN_FORWARD_STATIC_MAX_BYTES
            assert fits == (not (cid == 10 and M == 300))
            bnn.bnn_set_option(bnn.BNN_OPT_REALW_SPLIT_LOGSOFTMAX, 1 if fits else 0)
            try:
                want = model.forward(X)
            finally:
                bnn.bnn_set_option(bnn.BNN_OPT_REALW_SPLIT_LOGSOFTMAX, 1)
            got = torch.full((M, model.N_out), float("nan"), dtype=torch.float32, device=G.DEV)
            bnn.bnn_forward_static(model.layers, model.n_layers, G.ptr(X), M, G.ptr(got), G.stream())
            torch.cuda.synchronize()
            assert torch.isfinite(got).all()
            assert torch.equal(got.view(torch.int32), want.view(torch.int32)), (cfg.name, M)

    # a batch whose buffers do not fit the fixed array is refused, and nothing is enqueued
    cfg = workloads.CONFIGS[3]
    Ws, bs = workloads.make_net_params(cfg)
    model = G.GpuModel(Ws, bs, cfg.hidden_act, cfg.word_bits)
    M = 32768 + 64
    assert bnn.bnn_forward_workspace_bytes(model.layers, model.n_layers, M) > bnn.BNN_FORWARD_STATIC_MAX_BYTES
    with pytest.raises(bnn.BnnError) as e:
        bnn.bnn_forward_static(model.layers, model.n_layers, 0x10000, M, 0x20000, G.stream())
    assert e.value.status == bnn.BNN_EWORKSPACE
