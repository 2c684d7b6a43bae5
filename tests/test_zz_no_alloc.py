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

    for cid, batches in ((3, (1500, 333)), (8, (1100, 70)), (10, (300, 96)), (9, (600, 200))):
        cfg = workloads.CONFIGS[cid]
        Ws, bs = workloads.make_net_params(cfg)
        model = G.GpuModel(Ws, bs, cfg.hidden_act, cfg.word_bits, real_weight_layers=cfg.real_weight_layers)
        for M in batches:
            X = G.to_dev(workloads.make_frames(cfg, M))
            # Config 10 at 300 frames and Config 9 at 600: the extra scratch of the tiled matrix-core products (six bytes per
            # weight of Config 10's Softmax layer, a byte per weight of Config 9's real-input layers) does not fit the
            # fixed array, so the static entry point runs those layers on the kernels bnn_forward uses with these products
            # switched off
            fits = bnn.bnn_forward_workspace_bytes(model.layers, model.n_layers, M) <= bnn.BNN_FORWARD_STATIC_MAX_BYTES
            assert fits == ((cid, M) not in ((10, 300), (9, 600)))
            lean = ((bnn.BNN_OPT_REALW_SPLIT_LOGSOFTMAX, 0), (bnn.BNN_OPT_REALX_SIGN_MFMA, 2), (bnn.BNN_OPT_REALX_I8_LOGSOFTMAX, 2))
            if not fits:
                for opt, val in lean:
                    bnn.bnn_set_option(opt, val)
            try:
                want = model.forward(X)
            finally:
                for opt, _ in lean:
                    bnn.bnn_set_option(opt, 1)
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
