"""moss_quant_act_2level_noalloc (the entry point whose scratch is a static device array) gives the outputs of
moss_quant_act_2level bit for bit, on calls in a row that share the array: a tensor on the one-launch path, then a
smaller one on the two-launch path, then the first shape again."""
import numpy as np
import pytest
import torch

import moss_inputs as mi
import paper_2511_05811_amd as moss
from gpu_util import bf16_to_gpu

pytestmark = pytest.mark.gpu


def outputs(rows, cols, dev):
    u8 = torch.uint8
    return dict(q_row=torch.full((rows, cols), 0xAB, dtype=u8, device=dev), e_row=torch.full((rows, cols // 32), 0xAB, dtype=u8, device=dev),
                q_col=torch.full((cols, rows), 0xAB, dtype=u8, device=dev), e_col=torch.full((cols, rows // 32), 0xAB, dtype=u8, device=dev),
                s=torch.zeros(1, dtype=torch.float32, device=dev))


@pytest.mark.parametrize("flags", [moss.MOSS_Q_ROW | moss.MOSS_Q_COL, moss.MOSS_Q_ROW, moss.MOSS_Q_COL | moss.MOSS_EXP_CEIL])
def test_static_scratch_entry_point_matches_the_workspace_entry_point(flags):
    dev = torch.device("cuda:0")
    shapes = [(4096, 4096), (480, 1056), (4096, 4096), (64, 128)]      # second and fourth are smaller than the call before
    for i, (rows, cols) in enumerate(shapes):
        print(f"[no-alloc] flags={flags} call {i}: {rows}x{cols}", flush=True)
        x = bf16_to_gpu(mi.heavy_tailed_activation(rows, cols, seed=20 + i))
        want = moss.quant_act_2level(x, flags, out=outputs(rows, cols, dev))
        out = outputs(rows, cols, dev)
        n_alloc = torch.cuda.memory_stats()["allocation.all.allocated"]       # allocations torch has made so far
        got = moss.quant_act_2level_noalloc(x, flags, out)
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == n_alloc
        torch.cuda.synchronize()
        for k in ("q_row", "e_row", "q_col", "e_col", "s"):
            if want[k] is not None:          # (an output the flags do not ask for)
                assert torch.equal(got[k], want[k]), (i, k)
            else:
                assert bool((got[k] == 0xAB).all()), (i, k, "an output that was not asked for was written")
        assert float(got["s"]) > 0.0
