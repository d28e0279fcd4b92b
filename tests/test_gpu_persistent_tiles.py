"""Element-by-element parity of the bf16 block-contraction kernel on launches with more output tiles than resident
workgroups, so that every workgroup walks over several tiles: the next tile's addressing worked out under the
current one, its first stages issued before the current tile's epilogue, the two alternating sets of Z offset
tables.  The reduction is short (a stage or two per tile), which keeps the loop-nest oracle at a few seconds and
makes the per-tile phases, not the main loop, what the launch consists of.  Every case runs under all tile shapes
of the direct-to-LDS kernel and is compared with the oracle at every element (Section 4.3 of the paper: the
per-block kernel K over every join tuple, then the aggregation of the partial blocks)."""
import numpy as np
import pytest

from tests._parity import RTOL_BF16, RTOL_F32, single_vertex, tile_of, violations
from oracle.graph_ref import run_graph
from synth_inputs.prng import HostTensor, uniform_pm1

pytestmark = pytest.mark.gpu

# spec, bound X, bound Y, partitioning, result dtype; tiles of 256 x 256 / of 128 x 128 over all tuples
CASES = [
    # 18 x 18 = 324 large tiles with an 8-wide ragged edge (4360 = 17 * 256 + 8), 1225 small ones
    ("ij,jk->ik", (4360, 136), (136, 4360), {}, "f32"),
    ("ij,kj->ik", (4360, 136), (4360, 136), {}, "bf16"),
    ("ji,jk->ik", (136, 4360), (136, 4360), {}, "f32"),
    # the contracted label cut in two: every tile is written twice, into two partial slabs, and aggregated
    ("ij,jk->ik", (4360, 144), (144, 4360), {"j": 2}, "f32"),
    # rows and columns cut as well: 8 tuples, blocks of 2184 x 2184 (9 x 9 large tiles each, ragged), two slabs
    ("ij,jk->ik", (4368, 144), (144, 4368), {"i": 2, "j": 2, "k": 2}, "bf16"),
    # batched: 4 x 9 x 9 = 324 large tiles
    ("bij,bjk->bik", (4, 2200, 72), (4, 72, 2200), {}, "f32"),
    ("bij,bkj->bik", (4, 2200, 72), (4, 2200, 72), {"b": 2}, "bf16"),
    # 29 x 29 = 841 large tiles (more than three per workgroup), 3249 small ones
    ("ij,jk->ik", (7200, 72), (72, 7200), {}, "bf16"),
    ("ij,kj->ik", (7200, 72), (7200, 72), {}, "f32"),
]
_last = {}                                                   # the oracle's result for the case that ran last (the tile size varies fastest)


@pytest.mark.parametrize("tile", ["128", "256x128", "256"])
@pytest.mark.parametrize("spec,bx,by,part,out_dtype", CASES)
def test_bf16_contraction_with_several_tiles_per_workgroup(spec, bx, by, part, out_dtype, tile):
    import torch
    import paper_2410_02682_amd as E
    from paper_2410_02682_amd.runner import GraphRunner, to_device, to_host
    print(f"bf16 contraction {spec} X{bx} Y{by} d {part} -> {out_dtype}, tile {tile}", flush=True)
    x = HostTensor.from_f32(uniform_pm1(31, 0, int(np.prod(bx))).reshape(bx), "bf16")
    y = HostTensor.from_f32(uniform_pm1(31, 1, int(np.prod(by))).reshape(by), "bf16")
    w = single_vertex(spec, x, y, out_dtype, parts={"d": part})
    key = (spec, bx, by, tuple(sorted(part.items())), out_dtype)
    if _last.get("key") != key:
        _last.clear()
        _last.update(key=key, ref=run_graph(w, {"X": x, "Y": y})["Z"].as_f64())
    ref = _last["ref"]
    tm, tn = tile_of(tile)
    r = GraphRunner(w, "d", contract=dict(kernel="dma", tile=(tm, tn)))
    try:
        r.bind({"X": to_device(x), "Y": to_device(y)})
        pl = r.plan("Z")
        assert pl["kernel"] == "contract_mfma"
        # the launch must have more tiles than the chip holds workgroups of this kernel (one per compute unit for
        # the 256 x 256 tile, two for the others), or the case does not test what it is here for
        bz = pl["block_z"]                                   # Z is (b,) i, k in every case: batch entries, rows, columns of a block
        tiles = pl["n_tuples"] * int(np.prod(bz[:-2])) * (-(-bz[-2] // tm)) * (-(-bz[-1] // tn))
        cus = torch.cuda.get_device_properties(0).multi_processor_count
        assert tiles > (1 if tile == "256" else 2) * cus, (tiles, cus)
        E.tr_profile_enable(r.g, 4)
        r.run()
        torch.cuda.synchronize()
        assert [rec["kernel"] for rec in E.tr_profile_read(r.g) if rec["stage"] == "join"] == ["contract_mfma"]
        got = to_host(r.output("Z")).as_f64()
    finally:
        r.close()
    rtol, rep = (RTOL_BF16 if out_dtype == "bf16" else RTOL_F32), {}
    bad, worst = violations(got, ref, rtol, report=rep)
    assert bad == 0, f"{bad} elements out of tolerance (worst {worst:.2f}x)"
    # the plain relative error, without the rms term, on the elements that are not small against the tensor
    assert rep["strict_worst"] <= rtol, rep
