"""The measurement aids do what their declarations say: the copy copies, the matrix-core loop
reports the flop count of its launch and finishes."""
import numpy as np
import pytest
import torch

from paper_2603_18636_amd import svoo

pytestmark = pytest.mark.gpu


def test_copy_is_exact_and_counts_both_directions():
    host = np.random.default_rng(5).integers(-2 ** 31, 2 ** 31 - 1, (1 << 20) + 12, dtype=np.int32)
    src = torch.from_numpy(host).to("cuda:0")
    dst = torch.zeros_like(src)
    moved = svoo.microbench_copy(src, dst)
    torch.cuda.synchronize()
    assert moved == 2 * src.numel() * 4
    assert torch.equal(src, dst)
    with pytest.raises(ValueError):
        svoo.microbench_copy(src, dst[:-4])


@pytest.mark.parametrize("random_operands", [True, False])
def test_mfma_loop_reports_its_flops(random_operands):
    sink = torch.full((16 * 256,), float("nan"), dtype=torch.float32, device="cuda:0")
    flops = svoo.microbench_mfma_bf16(sink, 50, random_operands)
    torch.cuda.synchronize()
    assert flops == 16 * 4 * 50 * 16 * 2 * 32 * 32 * 16
    assert torch.isfinite(sink).all()
    if not random_operands:
        # every operand is 0.125: each accumulator holds 4 instructions x 50 iterations x 16 products
        assert torch.all(sink == 4 * 16 * 200 * 16 * 0.125 * 0.125)


def test_attention_tile_skeleton_runs_every_instantiated_subset():
    """The LDS-path microbenchmark launches, finishes and rejects the subsets it does not instantiate."""
    src = torch.randn((3 << 20,), device="cuda:0").to(torch.bfloat16)        # 6 MiB of tile-like data
    sink = torch.zeros((512 * 256,), dtype=torch.float32, device="cuda:0")
    for parts in (1, 2, 3, 4, 7, 8, 11, 15):
        svoo.microbench_attn_tile(parts, 3, src, sink)
    torch.cuda.synchronize()
    assert torch.isfinite(sink).all()
    with pytest.raises(svoo.SvooError):
        svoo.microbench_attn_tile(5, 3, src, sink)
    with pytest.raises(ValueError):
        svoo.microbench_attn_tile(1, 3, src[:1000], sink)
