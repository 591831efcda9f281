"""The whole layer under HIP graph capture.  No entry point allocates, synchronises or records a
memset, so a caller can capture the layer's launches once and replay them; every replay must give
the eager result bit for bit, also with other work on the GPU between the replays."""
import numpy as np
import pytest
import torch

import paper_2502_01776_amd as S
from workloads import get_config, make_qkv, sample_rows
from helpers import dev_i32, device_tile_lists

pytestmark = pytest.mark.gpu


def layer(sh, q, k, v, rows, t, labels, mse, ws, kt, vt, o, lists, static):
    if static:
        S.svg_profile_heads_static(sh, q, k, v, rows, t, labels, mse)
    else:
        S.svg_profile_heads(sh, q, k, v, rows, t, labels, mse, ws, ws.numel())
    S.svg_layout_kv_temporal(sh, k, v, kt, vt, labels)
    S.svg_sparse_attn_fwd_kv2(sh, q, k, v, kt, vt, o, labels, *lists)


@pytest.mark.parametrize("name, static", [("mid128", False), ("mid64", True)])
def test_whole_layer_replays_from_a_hip_graph(name, static):
    cfg = get_config(name)
    sh = S.shape_from_config(cfg)
    q, k, v = (x.cuda() for x in make_qkv(cfg))
    rows_np = sample_rows(cfg)
    rows, t = dev_i32(rows_np), len(rows_np)
    BH = sh.B * sh.H
    lists = device_tile_lists(sh)
    ws = torch.empty(S.svg_workspace_bytes(sh, t), dtype=torch.uint8, device="cuda")

    def buffers():
        return (torch.full((BH,), 255, dtype=torch.uint8, device="cuda"),
                torch.full((BH, 2), -1.0, dtype=torch.float32, device="cuda"),
                torch.empty_like(k), torch.empty_like(v), torch.full_like(q, float("nan")))

    labels_e, mse_e, kt_e, vt_e, o_e = buffers()
    layer(sh, q, k, v, rows, t, labels_e, mse_e, ws, kt_e, vt_e, o_e, lists, static)
    torch.cuda.synchronize()
    assert torch.isfinite(o_e.float()).all() and set(labels_e.cpu().tolist()) <= {0, 1}

    labels, mse, kt, vt, o = buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):           # one run on the capture stream before capturing
        layer(sh, q, k, v, rows, t, labels, mse, ws, kt, vt, o, lists, static)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        layer(sh, q, k, v, rows, t, labels, mse, ws, kt, vt, o, lists, static)
    for replay in range(3):
        # wipe what a replay has to produce, and keep the GPU busy with eager work of our own in between
        labels.fill_(255)
        mse.fill_(-1.0)
        o.fill_(float("nan"))
        scratch = torch.empty_like(q)
        S.svg_layout_fwd(sh, q, scratch, labels_e)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(labels, labels_e), f"replay {replay}: labels"
        assert torch.equal(mse.view(torch.int32), mse_e.view(torch.int32)), f"replay {replay}: MSE bits"
        assert torch.equal(o.view(torch.int16), o_e.view(torch.int16)), f"replay {replay}: output bits"
