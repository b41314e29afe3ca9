"""GPU parity of camera_gather_micro_experts (Algorithm 2, lines 10-13): pure data movement, so every
output byte must equal the oracle's gather of the same bit patterns."""
import numpy as np
import pytest
import torch

from oracle import camera_oracle as orc
from paper_2508_02322_amd import inputs

pytestmark = pytest.mark.gpu


def bits(t):
    """Bit patterns of a bf16 / float32 tensor as a numpy integer array (the oracle then moves integers)."""
    t = t.detach().cpu().contiguous()
    return (t.view(torch.int16) if t.dtype == torch.bfloat16 else t.view(torch.int32)).numpy()


def weights(n_experts, d_ff, d_model, dtype, seed, pad=0):
    """Random weights; pad > 0 leaves unused elements between experts (expert stride > d_ff * d_model)."""
    g = torch.Generator().manual_seed(seed)
    def one(shape):
        rows = shape[1] * shape[2] + pad
        full = torch.randn((n_experts, rows), generator=g).to(dtype)
        return full, full[:, :shape[1] * shape[2]].view(n_experts, shape[1], shape[2])
    return one((n_experts, d_ff, d_model)), one((n_experts, d_ff, d_model)), one((n_experts, d_model, d_ff))


def check(cam, Wg, Wu, Wd, index, count, index_base=0, align=1):
    """Runs the GPU gather on views of device copies and compares with the oracle, expert by expert; with a row
    alignment the rows of a W_down block are the oracle's, then zeros up to the next multiple of it."""
    dev = lambda pair: None if pair is None else pair[0].cuda()[:, :pair[1].shape[1] * pair[1].shape[2]].view(pair[1].shape)
    g_d, u_d, d_d = dev(Wg), dev(Wu), dev(Wd)
    idx_d = torch.as_tensor(np.asarray(index), dtype=torch.int32).cuda()
    cnt_d = None if count is None else torch.as_tensor(np.asarray(count), dtype=torch.int32).cuda()
    gate_out, up_out, down_out = cam.gather_micro_experts(g_d, u_d, d_d, idx_d, cnt_d, index_base, down_row_align=align)
    torch.cuda.synchronize()
    n_experts, d_ff, d_model = Wg[1].shape
    cnt = np.full(n_experts, d_ff) if count is None else np.asarray(count)
    o_gate, o_up, o_down = orc.gather_micro_experts(bits(Wg[1]), bits(Wu[1]), bits(Wd[1]), index, cnt, index_base)
    np.testing.assert_array_equal(bits(gate_out), o_gate)
    np.testing.assert_array_equal(bits(up_out), o_up)
    flat = bits(down_out)
    pos = 0
    for e in range(n_experts):
        ld = -(-int(cnt[e]) // align) * align
        block = flat[pos * d_model:(pos + ld) * d_model].reshape(d_model, ld)
        np.testing.assert_array_equal(block[:, :cnt[e]], o_down[e])
        assert not block[:, cnt[e]:].any()
        pos += ld


@pytest.mark.parametrize("dtype,n_experts,d_ff,d_model,pad", [
    (torch.bfloat16, 5, 200, 72, 0),        # small, vector path
    (torch.bfloat16, 3, 1001, 136, 8),      # d_ff not a multiple of 8: rows of W_down are not 16-byte aligned
    (torch.float32, 4, 130, 36, 4),         # float32, odd sizes, padded expert stride
    (torch.bfloat16, 2, 32768, 16, 0),      # the longest W_down row the kernel takes
    (torch.float32, 1, 16384, 8, 0),
])
def test_gather_after_select_matches_oracle(cam, dtype, n_experts, d_ff, d_model, pad):
    Wg, Wu, Wd = weights(n_experts, d_ff, d_model, dtype, seed=d_ff, pad=pad)
    n = n_experts * d_ff
    E = inputs.energy_like(n, seed=d_ff + 1)
    seg = [e * d_ff for e in range(n_experts + 1)]
    for ratio in (0.2, 0.6):
        keep, per, kept_idx, _ = cam.select_prune(E.cuda(), seg, ratio, want_idx=True)
        n_keep = n - orc.prune_count(ratio, n)
        idx = kept_idx[:n_keep].cpu().numpy()
        o_keep, o_per, o_idx, _ = orc.select_prune(E.numpy(), seg, ratio)
        np.testing.assert_array_equal(idx, o_idx)
        check(cam, Wg, Wu, Wd, idx, per.cpu().numpy())
        check(cam, Wg, Wu, Wd, idx, per.cpu().numpy(), align=64 if ratio < 0.5 else 8)   # zero-padded W_down rows


def test_gather_with_the_bit_allocation_permutation(cam):
    n_experts, d_ff, d_model = 6, 384, 64
    Wg, Wu, Wd = weights(n_experts, d_ff, d_model, torch.bfloat16, seed=11)
    E = inputs.energy_like(n_experts * d_ff, seed=12)
    seg = [e * d_ff for e in range(n_experts + 1)]
    _, _, perm = cam.alloc_bits(E.cuda(), seg, [3, 2, 1], [0.2, 0.6, 0.2], want_perm=True)
    check(cam, Wg, Wu, Wd, perm.cpu().numpy(), None)


def test_gather_degenerate_cases(cam):
    n_experts, d_ff, d_model = 4, 96, 40
    Wg, Wu, Wd = weights(n_experts, d_ff, d_model, torch.bfloat16, seed=21)
    everything = np.arange(n_experts * d_ff)
    check(cam, Wg, Wu, Wd, everything, np.full(n_experts, d_ff))                 # keep all: a copy
    check(cam, Wg, Wu, Wd, [2 * d_ff + 7], [0, 0, 1, 0])                         # one entry, empty experts around it
    check(cam, Wg, Wu, Wd, [2 * d_ff + 7], [0, 0, 1, 0], align=512)              # the same with the largest row alignment
    check(cam, Wg, Wu, Wd, 500 + everything[::3], [32] * n_experts, index_base=500)   # a group behind another one
    rev = np.concatenate([np.arange(e * d_ff, (e + 1) * d_ff)[::-1] for e in range(n_experts)])
    check(cam, Wg, Wu, Wd, rev, None)                                            # any order inside an expert
    # nothing kept: no launch, no error
    g_d = Wg[1].cuda()
    out = cam.gather_micro_experts(g_d, g_d, Wd[1].cuda(), torch.empty(0, dtype=torch.int32, device="cuda"),
                                   torch.zeros(n_experts, dtype=torch.int32, device="cuda"))
    assert out[0].shape == (0, d_model)


def test_gather_entries_outside_their_expert_give_zeros_and_outputs_can_be_skipped(cam):
    n_experts, d_ff, d_model = 3, 64, 24
    Wg, Wu, Wd = weights(n_experts, d_ff, d_model, torch.float32, seed=31)
    g_d, u_d, d_d = Wg[1].cuda(), Wu[1].cuda(), Wd[1].cuda()
    index = torch.tensor([3, 1000000, 64 + 5, -7, 128 + 9], dtype=torch.int32, device="cuda")   # entries 1 and 3 are bad
    count = torch.tensor([2, 2, 1], dtype=torch.int32, device="cuda")
    gate_out, up_out, down_out = cam.gather_micro_experts(g_d, u_d, d_d, index, count)
    torch.cuda.synchronize()
    want_rows = [Wg[1][0, 3], torch.zeros(d_model), Wg[1][1, 5], torch.zeros(d_model), Wg[1][2, 9]]
    for r, w in enumerate(want_rows):
        assert torch.equal(gate_out[r].cpu(), w)
    down = down_out.cpu()
    blk0 = down[:2 * d_model].view(d_model, 2)
    assert torch.equal(blk0[:, 0], Wd[1][0, :, 3]) and torch.equal(blk0[:, 1], torch.zeros(d_model))
    blk1 = down[2 * d_model:4 * d_model].view(d_model, 2)
    assert torch.equal(blk1[:, 0], Wd[1][1, :, 5]) and torch.equal(blk1[:, 1], torch.zeros(d_model))
    # only the down projection
    only_down = cam.gather_micro_experts(None, None, d_d, index, count)
    assert only_down[0] is None and only_down[1] is None and torch.equal(only_down[2].cpu(), down)
    # only the rows
    only_rows = cam.gather_micro_experts(g_d, u_d, None, index, count)
    assert only_rows[2] is None and torch.equal(only_rows[0], gate_out) and torch.equal(only_rows[1], up_out)


@pytest.mark.parametrize("name", ["deepseek-moe-16b", "qwen2-57b-a14b"])
def test_gather_full_size_layer(cam, name):
    """A whole layer of the benchmark shape: energies from the scoring path's own generator stand-in
    (random, the gather does not care), masks from the GPU select, every output byte against the oracle."""
    cfg = inputs.CONFIGS[name]
    layer = inputs.make_layer(cfg, 0, device="cuda")
    seg = inputs.segment_offsets(cfg)
    E = inputs.energy_like(cfg.n_micro, seed=77)
    keep, per, kept_idx, _ = cam.select_prune(E.cuda(), seg, 0.4, want_idx=True)
    n_keep = cfg.n_micro - orc.prune_count(0.4, cfg.n_micro)
    per_h, idx_h = per.cpu().numpy(), kept_idx[:n_keep].cpu().numpy()
    groups = [("W", cfg.n_experts, cfg.d_ff, 0)]
    if cfg.n_shared:
        groups.append(("Ws", cfg.n_shared, cfg.d_ff_shared, cfg.n_micro_routed))
    seg_pos, idx_pos = 0, 0
    for prefix, n_e, d_ff, base in groups:
        cnt = per_h[seg_pos:seg_pos + n_e]
        n_idx = int(cnt.sum())
        idx = idx_h[idx_pos:idx_pos + n_idx]
        Wg, Wu, Wd = layer[prefix + "_gate"], layer[prefix + "_up"], layer[prefix + "_down"]
        gate_out, up_out, down_out = cam.gather_micro_experts(
            Wg, Wu, Wd, kept_idx[idx_pos:idx_pos + n_idx], per[seg_pos:seg_pos + n_e], base)
        torch.cuda.synchronize()
        o_gate, o_up, o_down = orc.gather_micro_experts(bits(Wg), bits(Wu), bits(Wd), idx, cnt, base)
        np.testing.assert_array_equal(bits(gate_out), o_gate)
        np.testing.assert_array_equal(bits(up_out), o_up)
        flat, pos = bits(down_out), 0
        for e in range(n_e):
            np.testing.assert_array_equal(flat[pos * cfg.d_model:(pos + cnt[e]) * cfg.d_model].reshape(cfg.d_model, cnt[e]),
                                          o_down[e])
            pos += cnt[e]
        seg_pos += n_e
        idx_pos += n_idx
