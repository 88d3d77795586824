"""The measurement aid mrp_probe_lm_traffic: it only reads the packed LM head and reads / rewrites the
logit tile, so the logits must come back bit for bit, for every mode and ragged sizes; bad arguments are
refused before any launch."""
import numpy as np
import pytest
import torch

import mrp_inputs as mi
import paper_2605_18817_amd as mrp
from harness import dev_bits

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("d,V,M", [(256, 4096, 128), (512, 4100, 37), (256, 1028, 1)])
def test_probe_leaves_the_logits_unchanged(d, V, M):
    cfg = mi.config(0, d=d, V=V, B=M, L=1)
    ctx = mrp.MrpContext(d, V, M, 1)
    try:
        Wp = mrp.pack_weight(dev_bits(mi.lm_head(cfg)))
        z0 = mi.logits0(cfg)
        z = torch.from_numpy(z0).cuda()
        for mode in (0, 1, 2, 2):
            ctx.probe_lm_traffic(mode, M, Wp, z)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(z.cpu().numpy(), z0)
        assert ctx.poll_error() == 0
        # refused before any launch
        assert ctx.probe_lm_traffic(3, M, Wp, z, check=False) == -2
        assert ctx.probe_lm_traffic(-1, M, Wp, z, check=False) == -2
        assert ctx.probe_lm_traffic(2, 0, Wp, z, check=False) == -2
        assert ctx.probe_lm_traffic(2, 129, Wp, z, check=False) == -2
        assert ctx.probe_lm_traffic(2, M, None, z, check=False) == -1
        assert ctx.probe_lm_traffic(1, M, Wp, None, check=False) == -1
        assert ctx.probe_lm_traffic(0, M, Wp, None) == 0      # mode 0 never touches z
    finally:
        ctx.close()


def test_probe_refuses_sizes_its_kernel_does_not_cover():
    ctx = mrp.MrpContext(128, 1001, 8, 1)     # V % 4 != 0 and d % 256 != 0
    try:
        z = torch.zeros((8, 1001), dtype=torch.float32, device="cuda")
        w = torch.zeros(1024 * 128, dtype=torch.int16, device="cuda")
        assert ctx.probe_lm_traffic(2, 8, w, z, check=False) == -2
    finally:
        ctx.close()
