"""bitnet_quantize_weights_static (the entry point that allocates nothing: its scratch is a static device array of
the library) against bitnet_quantize_weights, through the C ABI: packed bytes and gamma bit for bit, on two calls in a
row, the second with a smaller input, in both packing formats."""
import numpy as np
import pytest

from paper_2402_17764_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.mark.parametrize("fmt", ["2bit", "trit5"])
def test_quantize_weights_static_matches_the_workspace_entry_point(gpu_lib, fmt):
    f = gpu_lib.PACK_2BIT if fmt == "2bit" else gpu_lib.PACK_TRIT5
    for (N, K, layer) in [(4096, 3200, 0), (250, 1040, 1), (33, 70, 2)]:      # each smaller than the one before
        print("[case] quantize_weights_static %s N=%d K=%d" % (fmt, N, K), flush=True)
        W = torch.from_numpy(synth.weights(N, K, config=0, layer=layer, tensor=31)).cuda()
        p_ref, g_ref = gpu_lib.quantize_weights(W, fmt=f)
        packed = torch.full((gpu_lib.packed_bytes(N, K, f),), 0xAA, dtype=torch.uint8, device="cuda")
        gamma = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
        gpu_lib.quantize_weights_static(W, packed, gamma, fmt=f)
        torch.cuda.synchronize()
        assert gamma.cpu().numpy().tobytes() == g_ref.cpu().numpy().tobytes()
        assert torch.equal(packed, p_ref)
