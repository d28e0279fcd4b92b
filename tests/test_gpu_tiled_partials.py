"""Tile-ordered partial slabs (tr_set_tiled_partials, on by default): a contraction on the direct-to-LDS kernel whose
blocks are whole output tiles stores its fp32 partial blocks in the order its accumulators lie in registers, and the
aggregation kernel that follows undoes the order (Section 4.3: join, then aggregation; Section 4.2: the aggregation
sums the tuples that share an output block).  The sums are the same in the same order, so the result must equal the
dense-slab path bit for bit, and it is compared with the oracle as well.  Every tile shape and wave count of the join
kernel, bf16 and fp32 operands and results, batch labels, several row / column labels, a swapped operand order, a
strided destination, a contraction the execution cuts further; shapes with ragged tiles or a long reduction per tile
must fall back to dense slabs."""
import numpy as np
import pytest

from tests._parity import RTOL_BF16, RTOL_F32, single_vertex, tile_of, violations
from oracle.graph_ref import run_graph
from synth_inputs.prng import HostTensor, uniform_pm1

pytestmark = pytest.mark.gpu

# spec, bound X, bound Y, partitioning, operand dtype, result dtype, tile ("" = the library's choice), waves, tiled expected
CASES = [
    ("ij,jk->ik", (512, 256), (256, 512), {"j": 2}, "bf16", "f32", "256", 0, True),
    ("ij,jk->ik", (512, 256), (256, 512), {"j": 4}, "bf16", "bf16", "256", 4, True),
    ("ij,jk->ik", (512, 256), (256, 512), {"j": 2}, "bf16", "bf16", "256x128", 0, True),
    ("ij,jk->ik", (512, 256), (256, 512), {"j": 8}, "bf16", "f32", "128", 0, True),
    ("ij,kj->ik", (768, 192), (512, 192), {"i": 3, "j": 3, "k": 2}, "bf16", "bf16", "", 0, True),       # 256 x 256 blocks, 3 slabs, 6 output blocks
    ("ji,jk->ik", (256, 512), (256, 256), {"j": 16}, "bf16", "f32", "", 0, True),
    ("ij,jk->ik", (256, 128), (128, 256), {"j": 2}, "f32", "f32", "128", 0, True),                       # fp32 operands
    ("ij,jk->ik", (512, 128), (128, 256), {"j": 2}, "f32", "f32", "256", 0, True),
    ("bij,bjk->bik", (3, 256, 128), (3, 128, 384), {"j": 2, "b": 3}, "bf16", "bf16", "128", 0, True),    # a batch label, cut
    ("bij,bjk->bik", (2, 256, 128), (2, 128, 256), {"j": 4}, "bf16", "f32", "256", 0, True),             # a batch label inside the block
    ("aij,jk->aik", (2, 128, 256), (256, 256), {"j": 2}, "bf16", "bf16", "256", 0, True),                # two row labels that fuse
    ("iaj,jkc->iakc", (64, 4, 256), (256, 2, 128), {"j": 2, "a": 2}, "bf16", "f32", "128", 0, True),     # several row and column labels
    ("ij,jk->ki", (256, 256), (256, 512), {"j": 2}, "bf16", "bf16", "256", 0, True),                     # the operands change places
    ("ij,jk->ik", (128, 16384), (16384, 128), {}, "bf16", "f32", "", 0, None),                           # the execution cuts the reduction itself (either layout)
    # a long reduction per tile (above 4096 the library keeps dense slabs, unless it cuts the reduction further itself, as here)
    ("ij,jk->ik", (256, 16384), (16384, 256), {"j": 2}, "bf16", "f32", "256", 0, None),
    # ragged tiles: dense slabs
    ("ij,jk->ik", (520, 256), (256, 512), {"j": 2}, "bf16", "f32", "256", 0, False),
    ("ij,jk->ik", (512, 256), (256, 392), {"j": 2}, "bf16", "f32", "128", 0, False),
]


def _run(w, x, y, tile, waves, tiled, out=None):
    import torch
    import paper_2410_02682_amd as E
    from paper_2410_02682_amd.runner import GraphRunner, to_device
    contract = dict(kernel="dma", tile=tile_of(tile), waves=waves) if tile else dict(kernel="dma")
    r = GraphRunner(w, "d", contract=contract, tiled_partials=tiled)
    try:
        r.bind({"X": to_device(x), "Y": to_device(y)}, outputs=out)
        E.tr_profile_enable(r.g, 8)
        r.run()
        torch.cuda.synchronize()
        rec = E.tr_profile_read(r.g)
        return r.output("Z").clone(), [(q["stage"], q["kernel"]) for q in rec]
    finally:
        r.close()


@pytest.mark.parametrize("spec,bx,by,part,in_dtype,out_dtype,tile,waves,expect", CASES)
def test_tile_ordered_partial_slabs_equal_dense_ones_bit_for_bit(spec, bx, by, part, in_dtype, out_dtype, tile, waves, expect):
    import torch
    from paper_2410_02682_amd.runner import to_host
    print(f"tile-ordered partials {spec} X{bx} Y{by} d {part} {in_dtype}->{out_dtype} tile {tile or 'default'} waves {waves}", flush=True)
    x = HostTensor.from_f32(uniform_pm1(47, 0, int(np.prod(bx))).reshape(bx), in_dtype)
    y = HostTensor.from_f32(uniform_pm1(47, 1, int(np.prod(by))).reshape(by), in_dtype)
    w = single_vertex(spec, x, y, out_dtype, parts={"d": part})
    tiled, launches_t = _run(w, x, y, tile, waves, True)
    dense, launches_d = _run(w, x, y, tile, waves, False)
    assert launches_d == [("join", "contract_mfma"), ("aggregate", "none")], launches_d
    if expect is not None:
        assert launches_t == [("join", "contract_mfma"), ("aggregate", "aggregate_tiles" if expect else "none")], launches_t
    assert torch.equal(tiled.view(torch.int16 if out_dtype == "bf16" else torch.int32), dense.view(torch.int16 if out_dtype == "bf16" else torch.int32))
    ref = run_graph(w, {"X": x, "Y": y})["Z"].as_f64()
    rtol = RTOL_BF16 if out_dtype == "bf16" else (RTOL_F32 if in_dtype == "f32" else RTOL_F32)
    bad, worst = violations(to_host(tiled).as_f64(), ref, rtol)
    assert bad == 0, f"{bad} elements out of tolerance (worst {worst:.2f}x)"


def test_tile_ordered_partials_into_a_strided_destination():
    """The destination is a view with padded rows inside a larger tensor: the aggregation kernel's row and column
    tables carry the destination's strides, and nothing outside the view is touched."""
    import torch
    print("tile-ordered partials into a strided view", flush=True)
    bx, by = (256, 512), (512, 384)
    x = HostTensor.from_f32(uniform_pm1(48, 0, int(np.prod(bx))).reshape(bx), "bf16")
    y = HostTensor.from_f32(uniform_pm1(48, 1, int(np.prod(by))).reshape(by), "bf16")
    w = single_vertex("ij,jk->ik", x, y, "f32", parts={"d": {"j": 4}})
    outs = []
    for tiled in (True, False):
        big = torch.full((300, 520), 7.0, dtype=torch.float32, device="cuda")
        view = big[20:276, 64:448]
        z, launches = _run(w, x, y, "128", 0, tiled, out={"Z": view})
        assert launches[1] == ("aggregate", "aggregate_tiles" if tiled else "none"), launches
        mask = torch.ones_like(big, dtype=torch.bool)
        mask[20:276, 64:448] = False
        assert bool((big[mask] == 7.0).all())
        outs.append(z)
    assert torch.equal(outs[0], outs[1])
