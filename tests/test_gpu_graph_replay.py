"""vit_encode_packed_graph against vit_encode_packed: the first call with a (buffers, shape) key runs the kernels as
they are, the second records them into a HIP graph, later ones replay it.  Every call, replays included, must give
the plain call's bits on whatever the input buffer holds at that moment; replays are interleaved with the
program's own eager work on other shapes and with synchronisations, and a second key lives beside the first."""
import numpy as np
import pytest

import gen
from parity_util import say

pytestmark = pytest.mark.gpu


def _bits(t):
    import torch

    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


@pytest.mark.parametrize("name", ["test_medium_bf16", "test_small_fp32"])
def test_graph_replays_match_the_plain_call_on_changing_inputs(name):
    import torch

    import paper_2502_00937_amd as V

    cfg = gen.get_config(name)  # local + global layers, CLS, two-layer projector
    enc = V.VitEncoder(cfg, gen.make_weights(cfg, seed=0), device=0)
    try:
        shapes = {"a": ([2, 1, 3, 1], [2, 0, 1, 1]), "b": ([1, 2], [1, 1])}
        keys = {}
        for k, (tpi, ipr) in shapes.items():
            to = np.concatenate([[0], np.cumsum(tpi)]).astype(np.int32)
            n_tok, out_dim, _, _ = enc.query(int(to[-1]), len(tpi))
            dt = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
            keys[k] = dict(to=to, ipr=ipr, px=torch.empty((int(to[-1]), cfg["channels"], cfg["image_size"], cfg["image_size"]),
                                                          device="cuda"),
                           out=torch.empty((n_tok, out_dim), dtype=dt, device="cuda"))
        other_to = np.array([0, 1, 2, 3], dtype=np.int32)  # eager work of a third shape between the graph calls
        other_px = torch.from_numpy(gen.make_pixels(cfg, 3, seed=99)).cuda()
        enc.encode(other_px, [3], other_to)  # sizes the cached workspace once: it must not move under the graphs
        for rnd in range(5):  # call 1 eager, call 2 records, calls 3-5 replay; the two keys alternate
            for k, c in keys.items():
                c["px"].copy_(torch.from_numpy(gen.make_pixels(cfg, int(c["to"][-1]), seed=10 * rnd + len(k) + ord(k))).cuda())
                want, rto_want = enc.encode(c["px"], c["ipr"], c["to"])
                c["out"].fill_(float("nan"))
                got, rto = enc.encode(c["px"], c["ipr"], c["to"], out=c["out"], graph=True)
                enc.encode(other_px, [3], other_to)
                torch.cuda.synchronize()
                assert got.data_ptr() == c["out"].data_ptr() and list(rto) == list(rto_want)
                same = torch.equal(_bits(got), _bits(want))
                say(f"    graph call {rnd + 1} of shape {k}: bitwise equal to the plain call = {same}")
                assert same
    finally:
        enc.close()


def test_graph_entry_point_keeps_at_most_eight_sequences_and_still_answers():
    """Ten keys in turn, three rounds: the least recently used sequence is replaced each time, so nothing is ever
    replayed, and every call must still be right."""
    import torch

    import paper_2502_00937_amd as V

    cfg = gen.get_config("test_small_bf16")
    enc = V.VitEncoder(cfg, gen.make_weights(cfg, seed=0), device=0)
    try:
        to = np.array([0, 1, 3], dtype=np.int32)
        px = torch.from_numpy(gen.make_pixels(cfg, 3, seed=5)).cuda()
        want, _ = enc.encode(px, [2], to)
        outs = [torch.empty_like(want) for _ in range(10)]
        for rnd in range(3):
            for o in outs:
                o.fill_(float("nan"))
                enc.encode(px, [2], to, out=o, graph=True)
            torch.cuda.synchronize()
            for o in outs:
                assert torch.equal(_bits(o), _bits(want))
    finally:
        enc.close()


def test_graph_entry_point_validates_like_the_plain_call():
    import torch

    import paper_2502_00937_amd as V

    cfg = gen.get_config("test_small_bf16")
    enc = V.VitEncoder(cfg, gen.make_weights(cfg, seed=0), device=0)
    try:
        n_tok, out_dim, out_bytes, ws_bytes = enc.query(2, 1)
        px = torch.zeros((2, cfg["channels"], cfg["image_size"], cfg["image_size"]), device="cuda")
        out = torch.empty((n_tok, out_dim), dtype=torch.bfloat16, device="cuda")
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        with pytest.raises(V.VitError) as e:
            V.vit_encode_packed_graph(enc.handle, px.data_ptr(), [1], [0, 2], out.data_ptr(), out_bytes - 2, ws.data_ptr(), ws_bytes, 0)
        assert e.value.status == V.binding.VIT_ECAPACITY
        with pytest.raises(V.VitError) as e:
            V.vit_encode_packed_graph(enc.handle, px.data_ptr(), [1], [0, 0], out.data_ptr(), out_bytes, ws.data_ptr(), ws_bytes, 0)
        assert e.value.status == V.binding.VIT_EINVAL
        rto = V.vit_encode_packed_graph(enc.handle, 0, [0, 0], [0], 0, 0, 0, 0, 0)  # text-only requests: a no-op
        assert list(rto) == [0, 0, 0]
    finally:
        enc.close()
