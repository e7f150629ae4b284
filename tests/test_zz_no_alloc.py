"""nova_winograd_conv2d_static (the entry point that allocates nothing: its workspace is a fixed
array inside the library's device image) against nova_winograd_conv2d on the same inputs.

Both run the same kernels on slabs of whole images, and a tile's result does not depend on which
slab it is in, so the two outputs are compared bit for bit.  Two calls in a row share the array:
the second one is smaller and runs on whatever the first left behind.
"""
import sys

import numpy as np
import pytest
import torch

from paper_2512_18453_amd import nova, synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def both_ways(t, x, w, K, flags):
    xd, wd = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
    U = nova.nova_filter_transform(t, wd)
    want = nova.nova_winograd_conv2d(t, xd, U, K, flags=flags)
    got = torch.full_like(want, float("nan"))
    nova.nova_winograd_conv2d_static(t, xd, U, K, got, flags=flags)
    torch.cuda.synchronize()
    return got.cpu().numpy(), want.cpu().numpy()


def test_static_workspace_call_equals_workspace_call_twice_in_a_row():
    assert nova.nova_static_workspace_bytes() == 64 << 20
    m = 8
    t = nova.nova_make_transforms(synth.point_set("nova", m), m, 3)
    # first call: 24 images whose V and M (about 100 MB) need two slabs of the 64 MiB array
    N, C, K, H, W = 24, 128, 128, 56, 56
    say(f"[case] static workspace, first call N={N} C={C} K={K} {H}x{W} F({m},3) fp16")
    assert nova.nova_conv2d_workspace_bytes(N, C, H, W, K, m, nova.NOVA_F16, 0, N) > nova.nova_static_workspace_bytes()
    x, w = synth.make_layer(N, C, K, H, W, seed=91, dtype="f16")
    got, want = both_ways(t, x, w, K, 0)
    assert np.isfinite(want).all() and np.array_equal(got, want)
    # second call, smaller, ragged, ReLU: runs on what the first call left in the array
    N, C, K, H, W = 3, 40, 33, 17, 23
    say(f"[case] static workspace, second call N={N} C={C} K={K} {H}x{W} F({m},3) fp16 relu")
    x, w = synth.make_layer(N, C, K, H, W, seed=92, dtype="f16", x_dist="normal")
    got, want = both_ways(t, x, w, K, nova.NOVA_FLAG_RELU)
    assert np.isfinite(want).all() and np.array_equal(got, want)
    # third: the few-channel path (no M) in binary32, F(4,3)
    t4 = nova.nova_make_transforms(synth.point_set("nova", 4), 4, 3)
    N, C, K, H, W = 2, 3, 20, 30, 26
    say(f"[case] static workspace, third call N={N} C={C} K={K} {H}x{W} F(4,3) fp32")
    x, w = synth.make_layer(N, C, K, H, W, seed=93, dtype="f32", x_dist="normal")
    got, want = both_ways(t4, x, w, K, 0)
    assert np.isfinite(want).all() and np.array_equal(got, want)


def test_static_workspace_refuses_an_image_that_does_not_fit():
    m = 8
    t = nova.nova_make_transforms(synth.point_set("nova", m), m, 3)
    N, C, K, H, W = 1, 512, 64, 224, 224          # V of one image: 100 * 784 * 512 * 2 B = 80 MB
    say("[case] static workspace, single image too large")
    assert nova.nova_conv2d_workspace_bytes(N, C, H, W, K, m, nova.NOVA_F16, 0, 1) > nova.nova_static_workspace_bytes()
    xd = torch.zeros((N, C, H, W), dtype=torch.float16, device=DEV)
    U = torch.zeros(nova.nova_filter_bytes(K, C, m, nova.NOVA_F16) // 2, dtype=torch.float16, device=DEV)
    y = torch.zeros((N, K, H, W), dtype=torch.float16, device=DEV)
    with pytest.raises(nova.NovaError) as info:
        nova.nova_winograd_conv2d_static(t, xd, U, K, y)
    assert info.value.code == -5                   # NOVA_ENOSPC
