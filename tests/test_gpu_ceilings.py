"""The measurement helpers that bench.py reports beside the datasheet peaks (they are not part of the einsum path): the
plain copy must copy, the read-mostly stream must combine its pieces as it says (exclusive-or of 16-byte vectors), the
register-resident loops must report their operation counts, and bad arguments must come back as errors, not launches."""
import pytest

pytestmark = pytest.mark.gpu


def test_copy_and_read_mostly_streams_move_what_they_say():
    import torch
    import paper_2410_02682_amd as E
    print("ceilings: copy and read-mostly streams", flush=True)
    n = 3 * 4096 + 16                                   # not a whole number of workgroups
    g = torch.Generator(device="cuda").manual_seed(5)
    src = torch.randint(0, 256, (16 * n,), dtype=torch.uint8, device="cuda", generator=g)
    dst = torch.zeros(n + 16, dtype=torch.uint8, device="cuda")
    s = torch.cuda.current_stream().cuda_stream
    E.eg_ceiling_copy(dst.data_ptr(), src.data_ptr(), n, s)
    torch.cuda.synchronize()
    assert torch.equal(dst[:n], src[:n]) and int(dst[n:].sum()) == 0
    for streams in (2, 8, 16):
        dst.zero_()
        E.eg_ceiling_read(dst.data_ptr(), src.data_ptr(), streams, n, s)
        torch.cuda.synchronize()
        want = src[:n].clone()
        for k in range(1, streams):
            want ^= src[k * n:(k + 1) * n]
        assert torch.equal(dst[:n], want) and int(dst[n:].sum()) == 0, streams
    for bad in (lambda: E.eg_ceiling_read(dst.data_ptr(), src.data_ptr(), 3, n, s),
                lambda: E.eg_ceiling_read(dst.data_ptr(), src.data_ptr(), 8, n + 8, s),
                lambda: E.eg_ceiling_read(dst.data_ptr() + 4, src.data_ptr(), 8, n, s),
                lambda: E.eg_ceiling_read(0, src.data_ptr(), 8, n, s),
                lambda: E.eg_ceiling_copy(dst.data_ptr(), src.data_ptr(), 8, s)):
        with pytest.raises(E.EgError):
            bad()


def test_register_resident_loops_report_their_operation_counts():
    import torch
    import paper_2410_02682_amd as E
    print("ceilings: register-resident loops", flush=True)
    sink = torch.zeros(64, dtype=torch.float32, device="cuda")
    s = torch.cuda.current_stream().cuda_stream
    assert E.eg_ceiling_mfma_bf16(sink.data_ptr(), 8, 2, 10, s) == 8 * 2 * 4 * 10 * 8 * 2 * 32 * 32 * 16
    assert E.eg_ceiling_mfma_bf16_random(sink.data_ptr(), 8, 10, s) == 8 * 4 * 10 * 16 * 2 * 32 * 32 * 16
    assert E.eg_ceiling_valu_f32(sink.data_ptr(), 8, 2, 10, s) == 8 * 2 * 256 * 10 * 64
    torch.cuda.synchronize()
    assert float(sink.abs().sum()) == 0.0               # the sink is never written
    with pytest.raises(E.EgError):
        E.eg_ceiling_mfma_bf16(sink.data_ptr(), 8, 3, 10, s)
    with pytest.raises(E.EgError):
        E.eg_ceiling_valu_f32(sink.data_ptr(), 0, 2, 10, s)
