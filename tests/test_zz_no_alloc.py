"""camera_select_prune_noalloc (static device scratch, no allocation in the call) against camera_select_prune:
two calls in a row through the C ABI, the second on a smaller input, so that what the first call left in the
shared scratch would show."""
import numpy as np
import pytest
import torch

from oracle import camera_oracle as orc
from paper_2508_02322_amd import binding, inputs

pytestmark = pytest.mark.gpu


def _segments(n, n_seg):
    cuts = sorted(set(int(round(i * n / n_seg)) for i in range(n_seg + 1)))
    cuts[0], cuts[-1] = 0, n
    return cuts


def test_noalloc_select_matches_select_prune():
    cam = binding.Camera(device=0)
    ref = binding.Camera(device=0)          # the existing entry point, on a context of its own
    for n, n_seg, ratio, seed in ((184320, 65, 0.4, 5), (20001, 7, 0.6, 6), (4096, 1, 0.0, 7), (777, 3, 1.0, 8)):
        print(f"no-alloc select: n_micro {n}, {n_seg} segments, ratio {ratio}", flush=True)
        E = inputs.energy_like(n, seed, device="cuda")
        seg = _segments(n, n_seg)
        keep = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
        per = torch.full((len(seg) - 1,), -1, dtype=torch.int32, device="cuda")
        kept_idx = torch.full((n,), -1, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        cam.select_prune_noalloc(E, seg, ratio, keep, per, kept_idx)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        r_keep, r_per, r_idx, _ = ref.select_prune(E, seg, ratio, want_idx=True)
        torch.cuda.synchronize()
        n_kept = int(r_per.sum())
        assert torch.equal(keep, r_keep) and torch.equal(per, r_per)
        assert torch.equal(kept_idx[:n_kept], r_idx[:n_kept])
        # and both against the oracle on the same float32 energies
        o_keep, o_per, o_idx, _ = orc.select_prune(E.cpu().numpy(), seg, ratio)
        np.testing.assert_array_equal(keep.cpu().numpy(), o_keep)
        np.testing.assert_array_equal(per.cpu().numpy(), o_per)
        np.testing.assert_array_equal(kept_idx.cpu().numpy()[:n_kept], o_idx)
    # beyond the static scratch: refused with a clear error, nothing launched
    big = torch.zeros((1 << 20) + 4, dtype=torch.float32, device="cuda")
    with pytest.raises(binding.CameraError) as exc:
        cam.select_prune_noalloc(big, [0, big.numel()], 0.5, torch.empty(big.numel(), dtype=torch.uint8, device="cuda"),
                                 torch.empty(1, dtype=torch.int32, device="cuda"))
    assert exc.value.code == -6 and "static scratch" in exc.value.message
    # the largest size it accepts
    n = 1 << 20
    E = inputs.energy_like(n, 9, device="cuda")
    keep = torch.empty(n, dtype=torch.uint8, device="cuda")
    per = torch.empty(4, dtype=torch.int32, device="cuda")
    seg = _segments(n, 4)
    cam.select_prune_noalloc(E, seg, 0.25, keep, per)
    r_keep, r_per, _, _ = ref.select_prune(E, seg, 0.25)
    torch.cuda.synchronize()
    assert torch.equal(keep, r_keep) and torch.equal(per, r_per)
    cam.close()
    ref.close()
