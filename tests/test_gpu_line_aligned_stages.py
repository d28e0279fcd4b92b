"""Blocks that start inside a 128-byte line of an operand contiguous along the contracted label (Section 4.3: the kernel
K runs on sub-tensors, wherever the partitioning vector's slices happen to start): the direct-to-LDS contraction kernel
then lays a tile's stages on that operand's lines, the first stage starting before the block's first k with those
elements not fetched, and tiles whose own offset needs one stage fewer run an empty last one.  Slices of 608 and 520
bf16 (every other block 64 bytes into a line; offsets 0, 16, ..., 112 bytes), fp32 slices, either or both operands
contiguous along k, a batch label, the operands as views that themselves start inside a line, and shapes where the rule
must not apply (rows that differ in their offsets) all have to match the oracle."""
import numpy as np
import pytest

from tests._parity import RTOL_BF16, RTOL_F32, single_vertex, tile_of, violations
from oracle.graph_ref import run_graph
from synth_inputs.prng import HostTensor, uniform_pm1

pytestmark = pytest.mark.gpu

# spec, bound X, bound Y, partitioning, operand dtype, result dtype, tile
CASES = [
    ("ij,jk->ik", (256, 8 * 608), (8 * 608, 256), {"j": 8}, "bf16", "f32", "256"),        # X's blocks 0 / 64 bytes into a line
    ("ij,jk->ik", (512, 8 * 520), (8 * 520, 384), {"j": 8}, "bf16", "bf16", "256"),       # offsets 0, 16, ..., 112 bytes
    ("ij,jk->ik", (256, 8 * 520), (8 * 520, 256), {"j": 8, "i": 2}, "bf16", "f32", "128"),
    ("ij,kj->ik", (256, 4 * 616), (384, 4 * 616), {"j": 4}, "bf16", "f32", "256"),        # both operands contiguous along j
    ("ji,kj->ik", (4 * 616, 256), (256, 4 * 616), {"j": 4}, "bf16", "bf16", "256"),       # only Y
    ("ij,jk->ik", (256, 4 * 300), (4 * 300, 256), {"j": 4}, "f32", "f32", "256"),         # fp32: slices of 1200 bytes
    ("bij,bjk->bik", (2, 256, 4 * 616), (2, 4 * 616, 256), {"j": 4}, "bf16", "f32", "256"),
    ("ij,jk->ik", (256, 2 * 8200), (2 * 8200, 256), {"j": 2}, "bf16", "f32", "256"),      # a long reduction, dense slabs
    ("ij,jk->ik", (256, 8 * 2616), (8 * 2616, 256), {"j": 8}, "bf16", "f32", "256"),      # 40.9 stages, offsets up to 112 bytes: one stage more
    ("ij,jk->ik", (256, 8 * 600), (8 * 600, 256), {"j": 8}, "bf16", "f32", "256"),        # rows 9600 bytes apart: offsets differ from row to row, no alignment
    ("ij,jk->ik", (256, 8 * 608), (8 * 608, 256), {"j": 8}, "bf16", "f32", "256x128"),    # half-depth stages: not laid on lines
]


def _run(w, dev_in, tile):
    import torch
    from paper_2410_02682_amd.runner import GraphRunner
    r = GraphRunner(w, "d", contract=dict(kernel="dma", tile=tile_of(tile)))
    try:
        r.bind(dev_in)
        r.run()
        torch.cuda.synchronize()
        return r.output("Z").clone()
    finally:
        r.close()


@pytest.mark.parametrize("spec,bx,by,part,in_dtype,out_dtype,tile", CASES)
def test_blocks_that_start_inside_a_line(spec, bx, by, part, in_dtype, out_dtype, tile):
    from paper_2410_02682_amd.runner import to_device, to_host
    print(f"line-aligned stages {spec} X{bx} Y{by} d {part} {in_dtype}->{out_dtype} tile {tile}", flush=True)
    x = HostTensor.from_f32(uniform_pm1(53, 0, int(np.prod(bx))).reshape(bx), in_dtype)
    y = HostTensor.from_f32(uniform_pm1(53, 1, int(np.prod(by))).reshape(by), in_dtype)
    w = single_vertex(spec, x, y, out_dtype, parts={"d": part})
    got = _run(w, {"X": to_device(x), "Y": to_device(y)}, tile)
    ref = run_graph(w, {"X": x, "Y": y})["Z"].as_f64()
    rtol = RTOL_BF16 if out_dtype == "bf16" else RTOL_F32
    bad, worst = violations(to_host(got).as_f64(), ref, rtol)
    assert bad == 0, f"{bad} elements out of tolerance (worst {worst:.2f}x)"


@pytest.mark.parametrize("lead_x,lead_y", [(8, 0), (24, 40), (0, 56)])
def test_operands_that_are_views_starting_inside_a_line(lead_x, lead_y):
    """X and Y are column ranges of wider tensors, so already the first block's rows start lead * 2 bytes into a line; what lies
    in front of the views (and would be fetched if the skipped elements of a first stage were not masked) is NaN."""
    import torch
    from paper_2410_02682_amd.runner import to_device, to_host
    print(f"line-aligned stages on views, X starts {lead_x} elements into a line, Y {lead_y}", flush=True)
    bx, by = (256, 4 * 640), (384, 4 * 640)
    x = HostTensor.from_f32(uniform_pm1(54, 0, int(np.prod(bx))).reshape(bx), "bf16")
    y = HostTensor.from_f32(uniform_pm1(54, 1, int(np.prod(by))).reshape(by), "bf16")
    w = single_vertex("ij,kj->ik", x, y, "f32", parts={"d": {"j": 4}})
    bigx = torch.full((bx[0], bx[1] + 128), float("nan"), dtype=torch.bfloat16, device="cuda")
    bigy = torch.full((by[0], by[1] + 128), float("nan"), dtype=torch.bfloat16, device="cuda")
    assert bigx.data_ptr() % 128 == 0 and bigy.data_ptr() % 128 == 0
    vx, vy = bigx[:, lead_x:lead_x + bx[1]], bigy[:, lead_y:lead_y + by[1]]
    vx.copy_(to_device(x))
    vy.copy_(to_device(y))
    got = _run(w, {"X": vx, "Y": vy}, "256")
    ref = run_graph(w, {"X": x, "Y": y})["Z"].as_f64()
    bad, worst = violations(to_host(got).as_f64(), ref, RTOL_F32)
    assert bad == 0, f"{bad} elements out of tolerance (worst {worst:.2f}x)"


@pytest.mark.parametrize("seed", range(24))
def test_random_slices_of_the_contracted_label_in_views(seed):
    """Seeded shapes: the contracted label cut 2, 4 or 8 ways into slices of 512 to 1400 elements (whole 16-byte chunks, any
    offset inside a line), the four operand layouts, bf16 and fp32, operands that are views starting 0 to 7 chunks into a
    line of tensors filled with NaN, rows a whole number of lines apart (so that the stages do get laid on lines), under
    the 256 x 256 tile, the 128 x 128 tile and the library's choice."""
    import random
    import torch
    from paper_2410_02682_amd.runner import GraphRunner, to_device, to_host
    r = random.Random(seed)
    dt = r.choice(["bf16", "bf16", "f32"])
    epc = 8 if dt == "bf16" else 4
    d = r.choice([2, 4, 8])
    kper = epc * r.randint(512 // epc, 1400 // epc)
    K, M, N = d * kper, r.choice([128, 256, 384]), r.choice([128, 256, 320])
    spec = r.choice(["ij,jk->ik", "ij,kj->ik", "ji,jk->ik", "ji,kj->ik"])
    bx = (M, K) if spec.startswith("ij") else (K, M)
    by = (K, N) if ",jk" in spec else (N, K)
    out_dt = r.choice(["f32", "bf16"]) if dt == "bf16" else "f32"
    lead_x, lead_y = epc * r.randint(0, 7), epc * r.randint(0, 7)
    print(f"random slices {seed}: {spec} X{bx} Y{by} {dt}->{out_dt} j cut {d} ways, views start {lead_x} / {lead_y} elements into a line", flush=True)
    x = HostTensor.from_f32(uniform_pm1(900 + seed, 0, int(np.prod(bx))).reshape(bx), dt)
    y = HostTensor.from_f32(uniform_pm1(900 + seed, 1, int(np.prod(by))).reshape(by), dt)
    w = single_vertex(spec, x, y, out_dt, parts={"d": {"j": d}})
    ref = run_graph(w, {"X": x, "Y": y})["Z"].as_f64()
    tdt = torch.bfloat16 if dt == "bf16" else torch.float32
    bigx = torch.full((bx[0], bx[1] + 64 + (-bx[1]) % 64), float("nan"), dtype=tdt, device="cuda")
    bigy = torch.full((by[0], by[1] + 64 + (-by[1]) % 64), float("nan"), dtype=tdt, device="cuda")
    vx, vy = bigx[:, lead_x:lead_x + bx[1]], bigy[:, lead_y:lead_y + by[1]]
    vx.copy_(to_device(x))
    vy.copy_(to_device(y))
    for tile in ("256", "128", ""):
        got = _run(w, {"X": vx, "Y": vy}, tile) if tile else None
        if got is None:
            rr = GraphRunner(w, "d")
            try:
                rr.bind({"X": vx, "Y": vy})
                rr.run()
                torch.cuda.synchronize()
                got = rr.output("Z").clone()
            finally:
                rr.close()
        bad, worst = violations(to_host(got).as_f64(), ref, RTOL_BF16 if out_dt == "bf16" else RTOL_F32)
        assert bad == 0, f"tile {tile or 'default'}: {bad} elements out of tolerance (worst {worst:.2f}x)"
