"""Bit-exact parity of the gfx950 library (through its C ABI) with the CPU oracle.

Every case draws seeded operands, runs the oracle on the host and the library on the
GPU, and compares element by element: integer work, so the bar is equality.
"""
import os
import zlib

import numpy as np
import pytest
import torch

from paper_2202_05239_amd import binding as f8
from paper_2202_05239_amd import workloads as wl

pytestmark = pytest.mark.gpu

DEV = "cuda"
NP_DTYPE = {"u8": np.uint8, "s8": np.int8, "s32": np.int32}


def host_threads():
    return max(1, min(16, os.cpu_count() or 1))


def gpu_layer(L, x, res=None, offset=0):
    """Run one layer description through the C ABI.  offset > 0 places x at an address
    that is only 1- or 4-byte aligned, to reach the narrow gather paths."""
    if offset:
        buf = torch.empty(x.size + 64, dtype=torch.uint8, device=DEV)
        xt = buf[offset:offset + x.size].view(f8.TORCH_DTYPE[L.x_type]).view(*x.shape)
        xt.copy_(torch.from_numpy(x))
    else:
        xt = torch.from_numpy(x).to(DEV)
    wt = torch.from_numpy(L.w).to(DEV) if L.w is not None else None
    bt = torch.from_numpy(L.bias).to(DEV) if L.bias is not None else None
    rt = torch.from_numpy(res).to(DEV) if res is not None else None
    B = x.shape[0]
    P, Q = L.out_hw
    if L.op == "gpool":
        y = torch.empty((B, L.Cout), dtype=f8.TORCH_DTYPE[L.y_type], device=DEV)
        f8.f8_global_pool_fixed(xt, y, L)
    elif L.op == "maxpool":
        y = torch.empty((B, P, Q, L.Cout), dtype=f8.TORCH_DTYPE[L.x_type], device=DEV)
        f8.f8_maxpool(xt, y, L.x_type, (L.R, L.S), (L.stride, L.stride), (L.pad, L.pad))
    else:
        y = torch.full((B, P, Q, L.Cout), 77, dtype=f8.TORCH_DTYPE[L.y_type], device=DEV)
        fn = f8.f8_conv2d_fixed if L.op == "conv" else f8.f8_dwconv_fixed
        fn(xt, wt, bt, y, L, (L.stride, L.stride), (L.pad, L.pad), rt)
    torch.cuda.synchronize()
    return y.cpu().numpy()


@pytest.fixture
def forced_variant():
    """Force one tile variant of the LDS-direct dense kernel for the length of a test."""
    yield lambda v: f8.f8_tuning_set("conv_variant", v)
    f8.f8_tuning_set("conv_variant", -1)


def assert_same(got, want, what=""):
    assert got.shape == want.shape and got.dtype == want.dtype, (what, got.shape, want.shape, got.dtype, want.dtype)
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        i = tuple(bad[0])
        raise AssertionError("%s: %d of %d differ; first at %s: gpu %d oracle %d" %
                             (what, len(bad), got.size, i, int(got[i]), int(want[i])))


# ------------------------------------------------------------------------- configs 0, 1, 2

def test_config0_gemm(oracle):
    x, L = wl.config0()
    want = oracle.gemm_fixed(x, L.w.reshape(64, 64), L.bias, L)
    xt, wt, bt = (torch.from_numpy(a).to(DEV) for a in (x, L.w.reshape(64, 64), L.bias))
    y = torch.empty((256, 64), dtype=torch.uint8, device=DEV)
    f8.f8_gemm_fixed(xt, wt, bt, y, L)
    torch.cuda.synchronize()
    assert_same(y.cpu().numpy(), want, "config0")
    assert 0.3 < (want == 0).mean() < 0.7 and want.max() > 100     # not a degenerate draw


def test_config1_conv3x3(oracle):
    x, L = wl.config1()                                             # full batch 32
    got = gpu_layer(L, x)
    parts = np.array_split(np.arange(x.shape[0]), host_threads())
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(host_threads()) as ex:
        outs = list(ex.map(lambda idx: oracle.conv2d_fixed(x[idx], L.w, L.bias, L, (1, 1), (1, 1)),
                           [p for p in parts if len(p)]))
    want = np.concatenate(outs)
    assert_same(got, want, "config1")
    assert (want == 192).mean() > 0.01 and want.max() == 192        # the clip level is exercised


@pytest.mark.parametrize("with_residual", [False, True])
def test_config2_mbv2_block(oracle, with_residual):
    x, net = wl.config2(with_residual=with_residual)                # batch 64
    want = oracle.run_network_parallel(net, x, host_threads(), keep_all=True)
    t = {0: x}
    for L in net.layers:                                            # single-layer entry points
        t[L.dst] = gpu_layer(L, t[L.src], t[L.res] if L.res >= 0 else None)
        assert_same(t[L.dst], want[L.dst], "config2 " + L.name)
    chain = f8.Chain(net, keep_all=True).prepare(x.shape[0])        # and the chain runner
    out = chain.run(torch.from_numpy(x).to(DEV))
    torch.cuda.synchronize()
    assert_same(out.cpu().numpy(), want[net.layers[-1].dst], "config2 chain")
    for L in net.layers[:-1]:
        assert_same(chain.tensor(L.dst).cpu().numpy(), want[L.dst], "config2 chain " + L.name)
    # with fusion on the block runs as one kernel: same bits, no intermediates
    fused = f8.Chain(net, fusion=True).prepare(x.shape[0])
    assert fused.layer_info(0, x.shape[0])[0] == "block_fused"
    out2 = fused.run(torch.from_numpy(x).to(DEV))
    torch.cuda.synchronize()
    assert_same(out2.cpu().numpy(), want[net.layers[-1].dst], "config2 fused block")
    assert fused.tensor(net.layers[0].dst) is None
    plain = f8.Chain(net).prepare(x.shape[0])
    assert plain.layer_info(0, x.shape[0])[0] != "block_fused"
    assert torch.equal(plain.run(torch.from_numpy(x).to(DEV)), out2)


# ------------------------------------------------------------------------- whole networks

def check_network(oracle, x, net, oracle_images, what, lean_is_smaller=True):
    """GPU runs the full batch; the oracle runs the listed images (images are independent)."""
    xt = torch.from_numpy(x).to(DEV)
    chain = f8.Chain(net, keep_all=True).prepare(x.shape[0])
    out = chain.run(xt)
    torch.cuda.synchronize()
    idx = np.asarray(oracle_images)
    want = oracle.run_network_parallel(net, np.ascontiguousarray(x[idx]), host_threads(), keep_all=True)
    for L in net.layers[:-1]:
        got = chain.tensor(L.dst).cpu().numpy()[idx]
        assert_same(got, want[L.dst], "%s layer %s" % (what, L.name))
        if L.dst2 > 0:
            got = chain.tensor(L.dst2).cpu().numpy()[idx]
            assert_same(got, want[L.dst2], "%s layer %s, second format" % (what, L.name))
    assert_same(out.cpu().numpy()[idx], want[net.layers[-1].dst], what + " logits")
    # the memory-reusing plan gives the same logits, and repeated runs are identical
    lean = f8.Chain(net).prepare(x.shape[0])
    a = lean.run(xt).clone()
    b = lean.run(xt)
    torch.cuda.synchronize()
    assert torch.equal(a, out) and torch.equal(b, out), what + " lean plan / rerun"
    # the tensors of the memory-reusing plan (the one bench.py times) that are still whole after
    # the run, against the oracle itself
    survivors = 0
    for L in net.layers[:-1]:
        t = lean.tensor(L.dst)
        if t is not None:
            survivors += 1
            assert_same(t.cpu().numpy()[idx], want[L.dst], "%s lean plan, layer %s" % (what, L.name))
    assert survivors > 0 or len(net.layers) < 3
    if lean_is_smaller:          # (a net of a few layers may have nothing to reuse)
        assert lean.workspace_bytes(x.shape[0]) < chain.workspace_bytes(x.shape[0])
    else:
        assert lean.workspace_bytes(x.shape[0]) <= chain.workspace_bytes(x.shape[0])
    # fused inverted-residual blocks (where the network has any): the same logits again
    fused = f8.Chain(net, fusion=True).prepare(x.shape[0])
    if any(fused.layer_info(i, x.shape[0])[0] == "block_fused" for i in range(len(net.layers))):
        c = fused.run(xt)
        torch.cuda.synchronize()
        assert torch.equal(c, out), what + " fused blocks"
    return out


def test_config3_resnet18(oracle):
    x, net = wl.config3()                                           # batch 64, 224x224x3
    out = check_network(oracle, x, net, list(range(0, 64, 4)), "config3")
    assert out.shape == (64, 1, 1, 1000) and out.dtype == torch.int32


def test_config4_resnet50(oracle):
    x, net = wl.config4()                                           # batch 256, 224x224x3
    imgs = [0, 1, 2, 3, 100, 101, 254, 255]
    out = check_network(oracle, x, net, imgs, "config4")
    assert out.shape == (256, 1, 1, 1000)


def full_batch_logits(oracle, x, net, what):
    """Every image of the batch: the logits of the memory-reusing chain (fused stem, paired 1x1
    layers, the two halves of the batch on two streams: the launch configuration bench.py times)
    against the oracle's, image by image; the one-stream run and a captured graph of the
    two-stream run, replayed with eager work in between, must give the same bits."""
    xt = torch.from_numpy(x).to(DEV)
    chain = f8.Chain(net, streams=2).prepare(x.shape[0])
    out = chain.run(xt)
    torch.cuda.synchronize()
    one = f8.Chain(net).prepare(x.shape[0]).run(xt)
    torch.cuda.synchronize()
    assert torch.equal(out, one), what + ": two streams differ from one"
    buf = torch.zeros_like(out)
    graph = chain.capture(xt, buf)
    for rep in range(3):
        buf.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(buf, out), what + ": replay %d of the two-stream graph differs" % rep
        chain.run(xt)                       # eager work between the replays
    got = out.cpu().numpy()
    step = 4 * host_threads()
    for i0 in range(0, x.shape[0], step):
        want = oracle.run_network_parallel(net, np.ascontiguousarray(x[i0:i0 + step]), host_threads())
        assert_same(got[i0:i0 + step], want, "%s logits of images %d.." % (what, i0))
        print("%s: images %d..%d match" % (what, i0, min(i0 + step, x.shape[0]) - 1), flush=True)


def test_config3_resnet18_every_image(oracle):
    x, net = wl.config3()                                           # batch 64, all 64 x 1000 logits
    full_batch_logits(oracle, x, net, "config3")


def test_config4_resnet50_every_image(oracle):
    x, net = wl.config4()                                           # batch 256, all 256 x 1000 logits
    full_batch_logits(oracle, x, net, "config4")


def test_mobilenet_v2_forward(oracle):
    """Beyond the five baseline configs: the whole fixed-point MobileNetV2 (stem, 17 inverted
    residual blocks with depthwise layers and signed linear bottlenecks, head, pool, classifier)."""
    x, net = wl.mobilenet_v2_forward(batch=64)                      # 224x224x3
    out = check_network(oracle, x, net, [0, 1, 2, 31, 32, 61, 62, 63], "mobilenet_v2")
    assert out.shape == (64, 1, 1, 1000) and out.dtype == torch.int32


def test_mobilenet_v1_forward(oracle):
    x, net = wl.mobilenet_v1_forward(batch=32)                      # 224x224x3
    out = check_network(oracle, x, net, [0, 1, 15, 16, 30, 31], "mobilenet_v1")
    assert out.shape == (32, 1, 1, 1000) and out.dtype == torch.int32


def test_resnet50_private_fractional_lengths(oracle):
    """Every block output written in two formats, one per child (Sec. 4.3): both copies of every
    such tensor, and everything downstream of them, against the oracle."""
    x, net = wl.resnet50_private_fl(batch=64)                       # 224x224x3
    assert sum(L.dst2 > 0 for L in net.layers) == 15
    out = check_network(oracle, x, net, [0, 1, 62, 63], "resnet50 private FL")
    assert out.shape == (64, 1, 1, 1000) and out.dtype == torch.int32


def test_weights_stationary_3x3_64(oracle):
    """The 3x3 64 -> 64 and 128 -> 128 stride-1 layers take a kernel of their own (weights in registers,
    input rows in LDS): image widths from 8 to 64, heights that leave ragged last tiles, one-row images,
    every input / output type, a shift of zero, clips inside the range."""
    rng = np.random.default_rng(640)
    # batches large enough for the library to pick this kernel (at least 768 blocks of 128 pixels at
    # 64 channels, of 64 pixels at 128)
    for C, B, H, W, xt, yt, shift, clip in ((64, 85, 56, 56, "u8", "u8", 9, None), (64, 2048, 13, 8, "s8", "s8", 7, (-50, 90)),
                                            (64, 2051, 1, 64, "u8", "s8", 8, None), (64, 1030, 7, 33, "s8", "u8", 0, (3, 200)),
                                            (64, 410, 31, 17, "u8", "u8", 11, (0, 1)), (64, 411, 9, 64, "u8", "u8", 6, None),
                                            (64, 256, 100, 9, "s8", "u8", 10, None), (64, 2, 56, 56, "u8", "u8", 9, None),
                                            (128, 158, 28, 28, "u8", "u8", 10, None), (128, 2048, 5, 8, "s8", "s8", 8, (-50, 90)),
                                            (128, 1030, 3, 38, "s8", "u8", 0, (3, 200)), (128, 700, 14, 14, "u8", "s8", 9, None),
                                            (128, 2049, 1, 33, "u8", "u8", 7, None), (128, 90, 47, 31, "s8", "u8", 11, (0, 1)),
                                            (128, 2, 28, 28, "u8", "u8", 10, None)):
        x, L, _ = wl.random_conv_case(rng, B, H, W, C, C, 3, 3, 1, 1, xt, yt, None, shift=shift, clip=clip)
        # images are independent: the single-threaded oracle runs on slices of the batch in host threads
        from concurrent.futures import ThreadPoolExecutor
        parts = np.array_split(np.arange(B), min(B, host_threads()))
        with ThreadPoolExecutor(len(parts)) as ex:
            outs = list(ex.map(lambda idx: oracle.conv2d_fixed(np.ascontiguousarray(x[idx]), L.w, L.bias, L, (1, 1), (1, 1)), parts))
        want = np.concatenate(outs)
        assert_same(gpu_layer(L, x), want, "ws 3x3 %s" % str((C, B, H, W, xt, yt, shift)))
    # in a chain the kernel's name shows: chosen at batch 256 of the full-size network, not for a few images
    _, net = wl.config4(batch=1)
    chain = f8.Chain(net)
    assert [chain.layer_info(i, 256)[0] for i in range(len(net.layers))].count("conv3x3_ws<64x64>") == 3
    assert [chain.layer_info(i, 2)[0] for i in range(len(net.layers))].count("conv3x3_ws<64x64>") == 0
    # (in a chain the 128-channel layers go to the image-stationary kernel unless that is switched off)
    f8.f8_tuning_set("conv_img", 0)
    try:
        chain = f8.Chain(net)
        assert [chain.layer_info(i, 256)[0] for i in range(len(net.layers))].count("conv3x3_ws<128x128>") == 3
    finally:
        f8.f8_tuning_set("conv_img", 1)


def test_image_stationary_3x3_256(oracle):
    """3x3 stride-1 layers with 256 -> 256 channels on images of at most 14 x 14 pixels, and with
    128 -> 128 channels on images at most 28 wide, take, in a chain with enough images to fill the CUs, a kernel
    that keeps one whole image in LDS and streams the weights (stored in fragment order when the
    workspace is prepared): image sizes with full, ragged and single blocks of pixels, batches
    below and above the number of workgroups, unsigned and signed inputs and outputs, clips inside
    the range; every image against the oracle, and against the general kernel."""
    for k, (C, hw, batch, x_type, relu1, relu2) in enumerate(((256, 14, 5, "u8", True, True), (256, 14, 300, "s8", True, False),
                                                               (256, 13, 257, "u8", False, True), (256, 7, 64, "u8", True, True),
                                                               (256, 3, 9, "s8", False, False), (256, 1, 2, "u8", True, True),
                                                               (128, 28, 5, "u8", True, True), (128, 28, 259, "s8", True, False),
                                                               (128, 27, 33, "u8", False, True), (128, 21, 17, "u8", True, True),
                                                               (128, 15, 70, "s8", False, False), (128, 2, 3, "u8", True, True))):
        rng = np.random.default_rng(1400 + k)
        b = wl._NetBuilder("img%d" % k, rng, hw, C, x_type, 5, (5, 9), (2, 6), True)
        a = b.conv("first", 0, C, 3, 1, 1, relu=relu1)
        b.conv("second", a, C, 3, 1, 1, relu=relu2)
        net = b.net
        x = wl.draw_u8(rng, (batch, hw, hw, C)) if x_type == "u8" else wl.draw_s8_normal(rng, (batch, hw, hw, C), 5)
        f8.f8_tuning_set("conv_img_min", 1)      # (also for fewer images than the kernel is normally chosen for)
        try:
            names = [f8.Chain(net).layer_info(i, batch)[0] for i in range(2)]
            assert names == ["conv3x3_img<%dx%d>" % (C, C)] * 2, names
            out = check_network(oracle, x, net, list(range(batch)), "image-stationary 3x3, case %d" % k, lean_is_smaller=False)
        finally:
            f8.f8_tuning_set("conv_img_min", 96)
        assert not any(f8.Chain(net).layer_info(i, 1)[0].startswith("conv3x3_img") for i in range(2))
        f8.f8_tuning_set("conv_img", 0)
        try:
            plain = f8.Chain(net).prepare(batch)
            assert not any(plain.layer_info(i, batch)[0].startswith("conv3x3_img") for i in range(2))
            other = plain.run(torch.from_numpy(x).to(DEV))
            torch.cuda.synchronize()
            assert torch.equal(other, out), "general kernel, case %d" % k
        finally:
            f8.f8_tuning_set("conv_img", 1)
    # the stride-1 3x3 layers of the full-size network's third (five) and second (three) stage
    _, net = wl.config4(batch=1)
    chain = f8.Chain(net)
    assert [chain.layer_info(i, 256)[0] for i in range(len(net.layers))].count("conv3x3_img<256x256>") == 5
    assert [chain.layer_info(i, 256)[0] for i in range(len(net.layers))].count("conv3x3_img<128x128>") == 3
    assert not any(chain.layer_info(i, 32)[0].startswith("conv3x3_img") for i in range(len(net.layers)))


def test_weights_stationary_1x1_64_to_256(oracle):
    """The 1x1 64 -> 256 layers at large batch take a kernel of their own (weights in registers, every
    wave streams 32-pixel blocks): with and without residual, residual scales above and below the
    accumulator's, every type combination, pixel counts that leave a ragged last block, a shift of
    zero, clips inside the range."""
    from concurrent.futures import ThreadPoolExecutor
    rng = np.random.default_rng(6400)
    for B, H, W, xt, yt, rt, shift, clip in ((43, 56, 56, "u8", "u8", "u8", 9, None), (2049, 8, 8, "s8", "s8", "s8", 7, (-50, 90)),
                                             (131073, 1, 1, "u8", "s8", None, 8, None), (1031, 7, 19, "s8", "u8", "u8", 0, (3, 200)),
                                             (410, 31, 11, "u8", "u8", "s8", 11, (0, 1)), (300, 21, 21, "u8", "u8", None, 6, None),
                                             (2, 56, 56, "u8", "u8", "u8", 9, None)):
        for rep in range(2 if rt else 1):      # two draws of the residual's fractional length
            x, L, res = wl.random_conv_case(rng, B, H, W, 64, 256, 1, 1, 1, 0, xt, yt, rt, shift=shift, clip=clip)
            parts = np.array_split(np.arange(B), min(B, host_threads()))
            with ThreadPoolExecutor(len(parts)) as ex:
                outs = list(ex.map(lambda idx: oracle.conv2d_fixed(np.ascontiguousarray(x[idx]), L.w, L.bias, L, (1, 1), (0, 0),
                                                                   None if res is None else np.ascontiguousarray(res[idx])), parts))
            assert_same(gpu_layer(L, x, res), np.concatenate(outs), "pw ws %s" % str((B, H, W, xt, yt, rt, shift, L.fl_res)))
    _, net = wl.config4(batch=1)
    chain = f8.Chain(net)
    # the shortcut projection; the three closing layers also compute the layer that opens the next block
    names = [chain.layer_info(i, 256)[0] for i in range(len(net.layers))]
    assert names.count("pw1x1_ws<64x256>") == 1 and names.count("pw1x1_ws<64x256>+1x1<64>") == 2
    assert names.count("pw1x1_ws<64x256>+1x1<128>") == 1
    assert not any(chain.layer_info(i, 4)[0].startswith("pw1x1_ws") for i in range(len(net.layers)))


def test_weights_stationary_1x1_256_and_512_inputs(oracle):
    """1x1 layers with 256 or 512 input channels and whole slices of output channels at large batch (the
    closing layers of the third and fourth ResNet stage) take a kernel whose waves keep the weights in
    registers: with and without residual, residual scales above and below the accumulator's, type
    combinations, pixel counts that leave a ragged last block, a shift of zero, clips inside the range."""
    from concurrent.futures import ThreadPoolExecutor
    rng = np.random.default_rng(25600)
    # (sizes from which the library picks this kernel: blocks of 32 pixels x channel slices >= 1024)
    for K, N, B, H, W, xt, yt, rt, shift, clip in ((256, 1024, 90, 14, 14, "u8", "u8", "u8", 10, None), (256, 1024, 531, 5, 13, "s8", "s8", "s8", 8, (-50, 90)),
                                                    (512, 2048, 131, 7, 7, "u8", "u8", "u8", 11, None), (512, 512, 2055, 1, 8, "u8", "s8", None, 9, None),
                                                    (256, 1024, 41, 19, 23, "s8", "u8", "s8", 0, (3, 200)), (512, 512, 271, 9, 7, "u8", "u8", "u8", 12, (0, 1)),
                                                    (512, 1024, 2, 112, 37, "u8", "u8", None, 10, None), (256, 2048, 33, 31, 9, "u8", "u8", "u8", 9, None)):
        for rep in range(2 if rt else 1):      # two draws of the residual's fractional length
            x, L, res = wl.random_conv_case(rng, B, H, W, K, N, 1, 1, 1, 0, xt, yt, rt, shift=shift, clip=clip)
            parts = np.array_split(np.arange(B), min(B, host_threads()))
            with ThreadPoolExecutor(len(parts)) as ex:
                outs = list(ex.map(lambda idx: oracle.conv2d_fixed(np.ascontiguousarray(x[idx]), L.w, L.bias, L, (1, 1), (0, 0),
                                                                   None if res is None else np.ascontiguousarray(res[idx])), parts))
            assert_same(gpu_layer(L, x, res), np.concatenate(outs), "pw wide %s" % str((K, N, B, H, W, xt, yt, rt, shift, L.fl_res)))
    _, net = wl.config4(batch=1)
    chain = f8.Chain(net)
    names = [chain.layer_info(i, 256)[0] for i in range(len(net.layers))]
    # the six closing layers of stage 3 and the three of stage 4
    assert names.count("pw1x1_wide<256>") == 6 and names.count("pw1x1_wide<512>") == 3, names
    assert not any(chain.layer_info(i, 4)[0].startswith("pw1x1_wide") for i in range(len(net.layers)))


def test_1x1_layer_computed_behind_the_64_to_256_layer(oracle):
    """A 1x1 64 -> 256 layer followed by a 1x1 256 -> 64 layer that reads its output (the hand-over
    between two bottleneck blocks): at large batch one launch computes both, the second from each
    block of the first one's output while it is on chip; both tensors are still written.  Every
    tensor against the oracle; the one-launch path against the two-launch path; small batches keep
    two launches."""
    cases = ((32, 128, 48, True, True, True, 64, False),     # unsigned in between, residual
             (23, 250, 16, False, True, False, 64, False),   # signed tensor in between, no residual, ragged last block
             (19, 370, 32, True, False, True, 128, False),   # 128 channels behind, signed output
             (37, 97, 16, False, False, True, 64, True),     # signed everywhere, ragged, another layer between the two
             (21, 300, 16, True, True, True, 128, True),     # the hand-over into a new stage: 128 channels, shortcut between
             (25, 210, 32, True, True, False, 128, False))   # 128 channels, no residual
    for k, (hw, batch, cin, relu1, relu2, with_res, cout2, between) in enumerate(cases):
        rng = np.random.default_rng(900 + k)
        b = wl._NetBuilder("tail%d" % k, rng, hw, cin, "u8", 6, (5, 9), (2, 6), True)
        r = b.conv("short", 0, 256, 1, 1, 0, relu=(k % 2 == 0))
        m = b.conv("mid", 0, 64, 1, 1, 0)
        h = b.conv("front", m, 256, 1, 1, 0, relu=relu1, res=r if with_res else -1)
        cj = 32 if between else cout2
        if between:      # (32 channels: this reader cannot itself be the layer computed behind the front one)
            e = b.conv("other_reader", h, cj, 1, 1, 0, relu=False)
            t = b.conv("behind", h, cout2, 1, 1, 0, relu=relu2)
        else:
            t = b.conv("behind", h, cout2, 1, 1, 0, relu=relu2)
            e = b.conv("other_reader", h, cj, 1, 1, 0, relu=False)
        b.conv("join", t, cj, 1, 1, 0, res=e)
        net = b.net
        x = wl.draw_u8(rng, (batch, hw, hw, cin))
        names = [f8.Chain(net).layer_info(i, batch)[0] for i in range(len(net.layers))]
        assert names[2] == "pw1x1_ws<64x256>+1x1<%d>" % cout2 and names[4 if between else 3] == "(fused)", names
        assert "(fused)" not in [f8.Chain(net).layer_info(i, 8)[0] for i in range(len(net.layers))]
        imgs = sorted(set([0, 1, batch // 2, batch - 2, batch - 1]))
        out = check_network(oracle, x, net, imgs, "1x1 behind 64->256, case %d" % k, lean_is_smaller=False)
        # the two-launch path: the same chain below the batch where one launch pays
        small = f8.Chain(net).prepare(8)
        xt = torch.from_numpy(x).to(DEV)
        for i0 in (0, batch - 8):
            part = small.run(xt[i0:i0 + 8].contiguous())
            torch.cuda.synchronize()
            assert torch.equal(part, out[i0:i0 + 8]), "two launches, case %d" % k


def test_1x1_layer_computed_behind_the_128_to_512_layer(oracle):
    """A 1x1 128 -> 512 layer followed by a 1x1 512 -> 128 layer that reads its output (the hand-over
    between two bottleneck blocks of the second stage): at large batch one launch computes both, the
    second from each block of the first one's output while it is on chip; both tensors are still
    written.  Every tensor against the oracle; the one-launch path against the two-launch path;
    small batches keep two launches."""
    cases = ((32, 64, True, True, True, False),      # unsigned in between, residual
             (23, 130, False, True, False, False),   # signed tensor in between, no residual, ragged last pair of blocks
             (19, 190, True, False, True, True),     # signed output, another layer between the two
             (37, 49, False, False, True, False))    # signed everywhere, ragged
    for k, (hw, batch, relu1, relu2, with_res, between) in enumerate(cases):
        rng = np.random.default_rng(1900 + k)
        b = wl._NetBuilder("tail128_%d" % k, rng, hw, 32, "u8", 6, (5, 9), (2, 6), True)
        r = b.conv("short", 0, 512, 1, 1, 0, relu=(k % 2 == 0))
        m = b.conv("mid", 0, 128, 1, 1, 0)
        h = b.conv("front", m, 512, 1, 1, 0, relu=relu1, res=r if with_res else -1)
        if between:      # (32 channels: this reader cannot itself be the layer computed behind the front one)
            e = b.conv("other_reader", h, 32, 1, 1, 0, relu=False)
            t = b.conv("behind", h, 128, 1, 1, 0, relu=relu2)
        else:
            t = b.conv("behind", h, 128, 1, 1, 0, relu=relu2)
            e = b.conv("other_reader", h, 32, 1, 1, 0, relu=False)
        b.conv("join", t, 32, 1, 1, 0, res=e)
        net = b.net
        x = wl.draw_u8(rng, (batch, hw, hw, 32))
        names = [f8.Chain(net).layer_info(i, batch)[0] for i in range(len(net.layers))]
        assert names[2] == "pw1x1_mid<128x512>+1x1<128>" and names[4 if between else 3] == "(fused)", names
        assert "(fused)" not in [f8.Chain(net).layer_info(i, 8)[0] for i in range(len(net.layers))]
        imgs = sorted(set([0, 1, batch // 2, batch - 2, batch - 1]))
        out = check_network(oracle, x, net, imgs, "1x1 behind 128->512, case %d" % k, lean_is_smaller=False)
        # the two-launch path: the same chain below the batch where one launch pays
        small = f8.Chain(net).prepare(8)
        xt = torch.from_numpy(x).to(DEV)
        for i0 in (0, batch - 8):
            part = small.run(xt[i0:i0 + 8].contiguous())
            torch.cuda.synchronize()
            assert torch.equal(part, out[i0:i0 + 8]), "two launches, case %d" % k
    # without the layer behind (switch at 2): the 128 -> 512 layer alone, through the single-layer call
    from concurrent.futures import ThreadPoolExecutor
    f8.f8_tuning_set("pw_mid", 2)
    try:
        rng = np.random.default_rng(1999)
        for B, H, W, xt_, yt, rt, shift, clip in ((70, 31, 31, "u8", "u8", "u8", 9, None), (1027, 8, 8, "s8", "s8", "s8", 7, (-50, 90)),
                                                  (65537, 1, 1, "u8", "s8", None, 0, (3, 100))):
            x, L, res = wl.random_conv_case(rng, B, H, W, 128, 512, 1, 1, 1, 0, xt_, yt, rt, shift=shift, clip=clip)
            parts = np.array_split(np.arange(B), min(B, host_threads()))
            with ThreadPoolExecutor(len(parts)) as ex:
                outs = list(ex.map(lambda idx: oracle.conv2d_fixed(np.ascontiguousarray(x[idx]), L.w, L.bias, L, (1, 1), (0, 0),
                                                                   None if res is None else np.ascontiguousarray(res[idx])), parts))
            assert_same(gpu_layer(L, x, res), np.concatenate(outs), "pw mid alone %s" % str((B, H, W, xt_, yt, rt, shift)))
    finally:
        f8.f8_tuning_set("pw_mid", 1)
    _, net = wl.config4(batch=1)
    chain = f8.Chain(net)
    assert [chain.layer_info(i, 256)[0] for i in range(len(net.layers))].count("pw1x1_mid<128x512>+1x1<128>") == 3


def test_weights_stationary_1x1_few_input_channels(oracle):
    """1x1 layers with 16, 24 or 32 input and 96, 144 or 192 output channels at large batch (MobileNetV2's
    first expand layers; also 32 -> 16, its first projection) take a streaming kernel of their own: every shape, input / output types,
    pixel counts that leave a ragged last block, a shift of zero, clips inside the range."""
    from concurrent.futures import ThreadPoolExecutor
    rng = np.random.default_rng(1696)
    for C, N, B, H, W, xt, yt, shift, clip in ((16, 96, 43, 56, 56, "s8", "u8", 8, None), (32, 144, 2049, 8, 8, "u8", "u8", 7, (3, 200)),
                                               (32, 192, 131073, 1, 1, "u8", "s8", 9, None), (16, 144, 1031, 7, 19, "s8", "s8", 0, (-50, 90)),
                                               (16, 192, 410, 31, 11, "u8", "u8", 10, (0, 1)), (32, 96, 300, 21, 21, "s8", "u8", 6, None),
                                               (24, 144, 45, 56, 56, "s8", "u8", 8, None), (24, 96, 1033, 127, 1, "u8", "s8", 7, (-100, 100)),
                                               (24, 192, 2050, 8, 8, "u8", "u8", 9, None), (32, 16, 47, 56, 56, "u8", "s8", 9, None),
                                               (32, 16, 131075, 1, 1, "s8", "u8", 6, (1, 77)), (32, 64, 83, 28, 29, "u8", "u8", 8, None), (16, 96, 2, 56, 56, "s8", "u8", 8, None)):
        x, L, _ = wl.random_conv_case(rng, B, H, W, C, N, 1, 1, 1, 0, xt, yt, None, shift=shift, clip=clip)
        parts = np.array_split(np.arange(B), min(B, host_threads()))
        with ThreadPoolExecutor(len(parts)) as ex:
            outs = list(ex.map(lambda idx: oracle.conv2d_fixed(np.ascontiguousarray(x[idx]), L.w, L.bias, L, (1, 1), (0, 0)), parts))
        assert_same(gpu_layer(L, x), np.concatenate(outs), "pw small %s" % str((C, N, B, H, W, xt, yt, shift)))
    # in the MobileNetV2 chain at batch 256: 16 -> 96, 24 -> 144 twice (read as they are, no padded copy), 32 -> 192 three times
    _, net = wl.mobilenet_v2_forward(batch=1)
    chain = f8.Chain(net)
    names = [chain.layer_info(i, 256)[0] for i in range(len(net.layers))]
    assert names.count("pw1x1_small<16x96>") == 1 and names.count("pw1x1_small<24x144>") == 2
    assert names.count("pw1x1_small<32x192>") == 3 and names.count("pw1x1_small<32x16>") == 1      # + the first projection
    assert not any(chain.layer_info(i, 2)[0].startswith("pw1x1_small") for i in range(len(net.layers)))


def test_fused_stem_and_pool(oracle):
    """The 7x7 stride-2 stem and the 3x3 stride-2 max pool behind it run as one kernel (when the
    tensor between them has no other reader): odd and tiny image sizes, ragged tiles, signed and
    unsigned images, a clip below 255, against the oracle and the two-kernel path."""
    for k, (hw, batch, x_type, hi) in enumerate(((31, 3, "s8", 255), (64, 2, "u8", 255), (75, 5, "s8", 140),
                                                 (113, 2, "u8", 201), (9, 4, "s8", 255), (224, 3, "s8", 255))):
        rng = np.random.default_rng(500 + k)
        b = wl._NetBuilder("stem%d" % hw, rng, hw, 3, x_type, 5, (5, 9), (2, 6), False)
        t = b.conv("conv1", 0, 64, 7, 2, 3)
        b.net.layers[-1].clip_hi = hi
        t = b.maxpool("maxpool", t)
        b.conv("head", t, 32, 1, 1, 0)
        net = b.net
        x = wl.draw_u8(rng, (batch, hw, hw, 3)) if x_type == "u8" else wl.draw_s8_normal(rng, (batch, hw, hw, 3), 5)
        want = oracle.run_network(net, x, keep_all=True)
        xt = torch.from_numpy(x).to(DEV)
        fused = f8.Chain(net).prepare(batch)
        assert fused.layer_info(0, batch)[0] == "stem_pool_fused"
        got = fused.run(xt)
        torch.cuda.synchronize()
        assert_same(got.cpu().numpy(), want[net.layers[-1].dst], "fused stem %d" % hw)
        assert fused.tensor(net.layers[0].dst) is None                   # never materialised
        assert_same(fused.tensor(net.layers[1].dst).cpu().numpy(), want[net.layers[1].dst], "pooled tensor %d" % hw)
        plain = f8.Chain(net, keep_all=True).prepare(batch)
        assert plain.layer_info(0, batch)[0] != "stem_pool_fused"
        assert torch.equal(plain.run(xt), got)
    # a second reader of the stem's output keeps the two kernels apart
    rng = np.random.default_rng(77)
    b = wl._NetBuilder("stem_two_readers", rng, 40, 3, "s8", 5, (5, 9), (2, 6), False)
    t = b.conv("conv1", 0, 64, 7, 2, 3)
    u = b.maxpool("maxpool", t)
    v = b.conv("side", t, 64, 3, 2, 1, relu=False)
    b.conv("join", u, 64, 1, 1, 0, res=v)
    x = wl.draw_s8_normal(rng, (2, 40, 40, 3), 5)
    chain = f8.Chain(b.net).prepare(2)
    assert chain.layer_info(0, 2)[0] != "stem_pool_fused"
    assert_same(chain.run(torch.from_numpy(x).to(DEV)).cpu().numpy(), oracle.run_network(b.net, x), "two readers")


def test_small_networks_full_compare(oracle):
    for cfg, batch in ((wl.config3, 5), (wl.config4, 3), (wl.mobilenet_v2_forward, 3), (wl.mobilenet_v1_forward, 2),
                       (wl.resnet50_private_fl, 3)):
        x, net = cfg(batch=batch, hw=64)
        check_network(oracle, x, net, list(range(batch)), net.name + " 64x64")


# ------------------------------------------------------------------------- layer sweeps

DENSE_CASES = [
    # B   H   W  Cin Cout R  S st pd  x     y     res    align-offset
    (2, 19, 23, 64, 64, 3, 3, 1, 1, "u8", "u8", None, 0),        # several 256-pixel tiles + ragged tail
    (3, 17, 17, 32, 160, 3, 3, 1, 1, "u8", "u8", "u8", 0),       # two N tiles, ragged N
    (2, 30, 14, 128, 128, 1, 1, 1, 0, "u8", "s8", "s8", 0),
    (2, 29, 31, 16, 24, 3, 3, 2, 1, "s8", "u8", None, 0),        # stride 2, N = 24
    (2, 33, 33, 64, 256, 1, 1, 2, 0, "u8", "s8", None, 0),       # downsample shortcut
    (1, 40, 40, 4, 64, 7, 7, 2, 3, "s8", "u8", None, 0),         # 4-byte gather path
    (2, 21, 21, 3, 32, 7, 7, 2, 3, "s8", "u8", None, 0),         # 1-byte gather path (C = 3)
    (1, 12, 13, 20, 10, 3, 3, 1, 1, "u8", "u8", "u8", 0),        # C % 4 == 0, N % 4 != 0
    (1, 9, 9, 7, 5, 3, 3, 1, 1, "u8", "s8", "s32", 0),           # odd everything
    (2, 10, 10, 48, 48, 3, 3, 1, 1, "u8", "u8", None, 4),        # x only 4-byte aligned
    (2, 10, 10, 48, 48, 3, 3, 1, 1, "u8", "u8", None, 1),        # x only 1-byte aligned
    (1, 1, 300, 512, 1000, 1, 1, 1, 0, "u8", "s32", None, 0),    # FC-like: int32 logits
    (1, 1, 7, 2048, 1000, 1, 1, 1, 0, "u8", "s32", "s32", 0),
    (1, 7, 7, 512, 512, 3, 3, 1, 1, "u8", "u8", "u8", 0),        # K = 4608
    (1, 5, 5, 8, 8, 5, 5, 1, 4, "u8", "u8", None, 0),            # padding wider than the image edge
    (1, 1, 1, 16, 16, 1, 1, 1, 0, "u8", "u8", None, 0),          # single pixel
    (1, 6, 6, 1, 1, 3, 3, 1, 1, "u8", "u8", None, 0),            # single channel in and out
    (4, 14, 14, 256, 64, 1, 1, 1, 0, "u8", "u8", "u8", 0),
    (2, 14, 14, 144, 24, 1, 1, 1, 0, "u8", "s8", "s8", 0),       # 1x1 with a partial last K step
    (2, 10, 11, 32, 144, 1, 1, 1, 0, "s8", "u8", None, 0),       # K shorter than one step, N = 144
    (1, 9, 9, 208, 80, 1, 1, 2, 0, "u8", "u8", None, 0),         # K = 13 x 16, strided 1x1
    (2, 6, 6, 96, 576, 1, 1, 1, 0, "u8", "u8", None, 0),
]


@pytest.mark.parametrize("case", DENSE_CASES)
def test_dense_layer_sweep(oracle, case):
    B, H, W, Cin, Cout, R, S, st, pd, xt, yt, rt, off = case
    rng = np.random.default_rng(zlib.crc32(repr(case).encode()))
    for trial in range(3):
        shift = [None, 0, -2][trial] if yt != "s32" else None
        x, L, res = wl.random_conv_case(rng, B, H, W, Cin, Cout, R, S, st, pd, xt, yt, rt, shift=shift)
        if trial == 1 and yt != "s32":
            L.clip_lo, L.clip_hi = (10, 100) if yt == "u8" else (-50, 60)
        want = oracle.conv2d_fixed(x, L.w, L.bias, L, (st, st), (pd, pd), res)
        got = gpu_layer(L, x, res, off)
        assert_same(got, want, "dense %s trial %d" % (str(case), trial))


def test_residual_shift_directions(oracle):
    """Residual finer than, equal to and coarser than the accumulator scale."""
    rng = np.random.default_rng(77)
    for fl_res in (0, 5, 9, 12, 14):
        x, L, res = wl.random_conv_case(rng, 2, 12, 12, 32, 32, 3, 3, 1, 1, "u8", "u8", "s8", shift=6)
        L.fl_x, L.fl_w, L.fl_y, L.fl_res = 4, 5, 3, fl_res
        want = oracle.conv2d_fixed(x, L.w, L.bias, L, (1, 1), (1, 1), res)
        assert_same(gpu_layer(L, x, res), want, "fl_res %d" % fl_res)


def test_shift_extremes(oracle):
    rng = np.random.default_rng(78)
    for shift, fl in ((24, (12, 12, 0)), (-8, (0, 0, 8)), (1, (1, 0, 0))):
        x, L, _ = wl.random_conv_case(rng, 1, 8, 8, 64, 32, 3, 3, 1, 1, "u8", "u8", shift=shift,
                                      w_std=30.0 if shift > 8 else 0.7)
        L.fl_x, L.fl_w, L.fl_y = fl
        if shift == 24:
            L.bias = rng.integers(0, 2 ** 30, L.Cout).astype(np.int32)
        want = oracle.conv2d_fixed(x, L.w, L.bias, L, (1, 1), (1, 1))
        assert_same(gpu_layer(L, x), want, "shift %d" % shift)
        assert len(np.unique(want)) > (1 if shift < 0 else 2)


def test_degenerate_inputs(oracle):
    rng = np.random.default_rng(79)
    x, L, _ = wl.random_conv_case(rng, 1, 8, 8, 16, 16, 3, 3, 1, 1)
    L.w[:] = 0                                                  # output = fix_quant(bias)
    assert_same(gpu_layer(L, x), oracle.conv2d_fixed(x, L.w, L.bias, L, (1, 1), (1, 1)), "zero weights")
    x, L, _ = wl.random_conv_case(rng, 1, 8, 8, 16, 16, 3, 3, 1, 1)
    L.clip_lo = L.clip_hi = 9                                   # degenerate clip
    assert (gpu_layer(L, x) == 9).all()
    x, L, _ = wl.random_conv_case(rng, 1, 8, 8, 16, 16, 1, 1, 1, 0, x_type="s8")
    x[:] = -128                                                 # -128 is accepted on input
    L.bias = None
    assert_same(gpu_layer(L, x), oracle.conv2d_fixed(x, L.w, None, L), "minus 128 input, no bias")
    x, L, _ = wl.random_conv_case(rng, 1, 8, 8, 16, 16, 1, 1, 1, 0)
    x[:] = 255
    L.w[:] = 127                                                # largest products
    assert_same(gpu_layer(L, x), oracle.conv2d_fixed(x, L.w, L.bias, L), "max magnitude")
    # empty batch: nothing launched, nothing written
    import ctypes
    y = torch.full((1, 8, 8, 16), 5, dtype=torch.uint8, device=DEV)
    xt, wt = torch.from_numpy(x).to(DEV), torch.from_numpy(L.w).to(DEV)
    q = f8.make_quant(L)
    rc = f8.lib().f8_conv2d_fixed(xt.data_ptr(), wt.data_ptr(), None, y.data_ptr(), 0, 8, 8, 16, 16, 1, 1,
                                  1, 1, 0, 0, ctypes.byref(q), None)
    torch.cuda.synchronize()
    assert rc == 0 and (y == 5).all()


DW_CASES = [
    (2, 19, 23, 144, 3, 3, 1, 1, "u8", "u8", None),
    (2, 20, 21, 96, 3, 3, 2, 1, "u8", "u8", None),
    (1, 15, 15, 32, 5, 5, 1, 2, "s8", "s8", "s8"),
    (1, 9, 11, 7, 3, 3, 1, 1, "u8", "u8", "u8"),           # channels not a multiple of 4
    (1, 8, 8, 24, 3, 3, 1, 0, "u8", "s32", None),
    (3, 7, 7, 576, 3, 3, 1, 1, "u8", "u8", None),
    (2, 17, 13, 36, 3, 3, 2, 1, "s8", "u8", None),         # stride 2, ragged strips and row chunks
    (1, 30, 9, 20, 3, 3, 1, 0, "s8", "s8", None),          # no padding, several row chunks
    (2, 33, 10, 8, 3, 3, 2, 0, "u8", "s8", None),
    (1, 3, 3, 4, 3, 3, 1, 1, "u8", "u8", None),            # image as small as the window
    (1, 12, 12, 16, 3, 3, 1, 2, "u8", "u8", None),         # padding wider than the usual 1
    (2, 14, 14, 64, 3, 3, 1, 1, "u8", "u8", "s8"),         # residual: generic kernel
]


@pytest.mark.parametrize("case", DW_CASES)
def test_depthwise_sweep(oracle, case):
    B, H, W, C, R, S, st, pd, xt, yt, rt = case
    rng = np.random.default_rng(zlib.crc32(repr(case).encode()))
    for trial in range(3):
        shift = [None, 0, -1][trial] if yt != "s32" else None
        x, L, res = wl.random_conv_case(rng, B, H, W, C, C, R, S, st, pd, xt, yt, rt, shift=shift, depthwise=True)
        want = oracle.dwconv_fixed(x, L.w, L.bias, L, (st, st), (pd, pd), res)
        assert_same(gpu_layer(L, x, res), want, "dw %s trial %d" % (str(case), trial))


def test_pools(oracle):
    rng = np.random.default_rng(80)
    for kind, shape, k, st, pd in (("u8", (2, 31, 29, 64), 3, 2, 1), ("s8", (1, 10, 10, 6), 2, 2, 0),
                                   ("u8", (1, 7, 9, 5), 3, 1, 1), ("s8", (2, 13, 17, 32), 3, 2, 1),
                                   ("s8", (1, 8, 8, 16), 2, 2, 0), ("u8", (3, 6, 5, 48), 3, 1, 1),
                                   ("s8", (1, 9, 9, 16), 3, 3, 0)):
        if kind == "u8":
            x = wl.draw_u8(rng, shape)
        elif shape[3] == 6:
            x = rng.integers(-128, 0, shape, dtype=np.int8)          # all negative: padding must never win
        else:
            x = rng.integers(-128, 128, shape, dtype=np.int8)
        want = oracle.maxpool(x, kind, (k, k), (st, st), (pd, pd))
        L = wl.LayerSpec(op="maxpool", Cin=shape[3], Cout=shape[3], R=k, S=k, stride=st, pad=pd,
                         x_type=kind, y_type=kind, out_hw=want.shape[1:3])
        assert_same(gpu_layer(L, x), want, "maxpool " + kind)
    for shape, fl_w in (((3, 7, 7, 512), 6), ((2, 5, 6, 10), 5), ((1, 2, 2, 3), 0)):
        x = wl.draw_u8(rng, shape)
        L = wl.LayerSpec(op="gpool", Cin=shape[3], Cout=shape[3], fl_x=4, fl_w=fl_w, fl_y=4, clip_lo=0,
                         clip_hi=255, x_type="u8", y_type="u8")
        assert_same(gpu_layer(L, x), oracle.global_pool_fixed(x, L), "gpool")


def test_repeatable_and_streams(oracle):
    """Same inputs, three runs, two streams: identical bits (the race detector)."""
    x, L = wl.config1(batch=4)
    xt, wt, bt = (torch.from_numpy(a).to(DEV) for a in (x, L.w, L.bias))
    want = oracle.conv2d_fixed(x, L.w, L.bias, L, (1, 1), (1, 1))
    outs = []
    s2 = torch.cuda.Stream()
    for i in range(3):
        y = torch.empty((4, 56, 56, 64), dtype=torch.uint8, device=DEV)
        if i == 1:
            s2.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(s2):
                f8.f8_conv2d_fixed(xt, wt, bt, y, L, (1, 1), (1, 1))
            s2.synchronize()
        else:
            f8.f8_conv2d_fixed(xt, wt, bt, y, L, (1, 1), (1, 1))
        torch.cuda.synchronize()
        outs.append(y.cpu().numpy())
    for o in outs:
        assert_same(o, want, "repeat")


def test_caller_workspace_entry_point_from_two_threads_and_streams(oracle):
    """f8_conv2d_fixed_ws keeps no state in the library: four host threads, each with its own stream
    and workspace, issue different layers at the same time, repeatedly; every result is the
    oracle's.  The allocating entry point, called from the same threads on one shared stream,
    must also stay correct (its scratch look-up and launches are under one lock)."""
    import threading
    rng = np.random.default_rng(4242)
    cases = [(2, 19, 23, 64, 72, 1, 1, 1, 0, "u8", "u8", "u8"), (1, 21, 9, 256, 40, 3, 3, 2, 1, "u8", "s8", None),
             (2, 15, 17, 32, 272, 3, 3, 1, 1, "u8", "u8", "s8"), (3, 13, 11, 128, 136, 1, 1, 1, 0, "s8", "s8", None)]
    jobs = []
    for case in cases:
        B, H, W, Cin, Cout, R, S, st, pd, xt, yt, rt = case
        x, L, res = wl.random_conv_case(rng, B, H, W, Cin, Cout, R, S, st, pd, xt, yt, rt)
        want = oracle.conv2d_fixed(x, L.w, L.bias, L, (st, st), (pd, pd), res)
        dev = [torch.from_numpy(a).to(DEV) if a is not None else None for a in (x, L.w, L.bias, res)]
        ws = torch.empty(f8.lib().f8_conv_workspace_bytes(Cout) + 256, dtype=torch.uint8, device=DEV)
        ws = ws[(-ws.data_ptr()) % 256:][:f8.lib().f8_conv_workspace_bytes(Cout)]
        jobs.append((L, dev, want, ws, torch.cuda.Stream(), (st, st), (pd, pd)))
    torch.cuda.synchronize()
    errors = []

    def worker(job, shared):
        L, (xd, wd, bd, rd), want, ws, stream, stride, pad = job
        try:
            for rep in range(6):
                y = torch.full(want.shape, 77, dtype=f8.TORCH_DTYPE[L.y_type], device=DEV)
                if shared:
                    f8.f8_conv2d_fixed(xd, wd, bd, y, L, stride, pad, rd)        # all threads on the default stream
                    torch.cuda.synchronize()
                else:
                    with torch.cuda.stream(stream):
                        y.fill_(77)
                        f8.f8_conv2d_fixed_ws(xd, wd, bd, y, L, ws, stride, pad, rd, stream=stream)
                    stream.synchronize()
                if not np.array_equal(y.cpu().numpy(), want):
                    errors.append((L.Cout, rep, shared))
        except Exception as e:                       # noqa: BLE001 (reported below)
            errors.append(repr(e))

    for shared in (False, True):
        threads = [threading.Thread(target=worker, args=(j, shared)) for j in jobs]
        for t in threads:
            t.start()
        for t in threads:
            t.join()
    assert not errors, errors
    # validation of the workspace arguments happens before any launch
    L, (xd, wd, bd, rd), want, ws, stream, stride, pad = jobs[0]
    y = torch.empty(want.shape, dtype=torch.uint8, device=DEV)
    with pytest.raises(f8.F8Error) as e:
        f8.f8_conv2d_fixed_ws(xd, wd, bd, y, L, ws[:64], stride, pad, rd)
    assert e.value.code == 2


# ------------------------------------------------------------------------- tile variants

N_TILE_VARIANTS = 24
SINGLE_STAGE = {8: 64, 9: 128, 10: 64}          # variants that hold the whole K in one step


@pytest.mark.parametrize("variant", range(N_TILE_VARIANTS))
def test_every_tile_variant(oracle, variant, forced_variant):
    """The tile choice is a tuning decision, never a numerical one: every tile variant of the
    fast dense kernel, forced through the tuning knob, gives the oracle's bits on ragged
    shapes (tails in M, N and K, padding, stride, residual, both K-step widths)."""
    forced_variant(variant)
    kmax = SINGLE_STAGE.get(variant)
    cases = [
        (2, 19, 23, 64, 72, 1, 1, 1, 0, "u8", "u8", "u8"),           # K = 64: one step for everyone
        (3, 13, 11, 128, 136, 1, 1, 1, 0, "s8", "s8", None),         # K = 128
        (2, 7, 9, 48, 20, 1, 1, 1, 0, "u8", "u8", "u8"),             # K = 48: partial step
    ]
    if kmax is None:
        cases += [
            (2, 15, 17, 32, 272, 3, 3, 1, 1, "u8", "u8", "s8"),      # K = 288, three N tiles of 128
            (1, 21, 9, 256, 40, 3, 3, 2, 1, "u8", "s8", None),       # K = 2304, stride 2
            (2, 9, 9, 384, 520, 1, 1, 1, 0, "u8", "u8", None),       # 128-byte lines, ragged N
            (2, 11, 5, 144, 24, 1, 1, 1, 0, "u8", "s8", "s8"),       # 1x1, K = 144: partial last step
            (1, 9, 9, 208, 80, 1, 1, 2, 0, "s8", "u8", None),
        ]
    rng = np.random.default_rng(1000 + variant)
    for case in cases:
        B, H, W, Cin, Cout, R, S, st, pd, xt, yt, rt = case
        if kmax is not None and R * S * Cin > kmax:
            continue
        x, L, res = wl.random_conv_case(rng, B, H, W, Cin, Cout, R, S, st, pd, xt, yt, rt)
        want = oracle.conv2d_fixed(x, L.w, L.bias, L, (st, st), (pd, pd), res)
        assert_same(gpu_layer(L, x, res), want, "variant %d case %s" % (variant, str(case)))


# ------------------------------------------------------------------------- two output formats

DUAL_CASES = [
    # B   H   W  Cin Cout R  S st pd  x     y     y2    res   shift shift2  offset of y2
    (2, 19, 23, 64, 72, 1, 1, 1, 0, "u8", "u8", "u8", "u8", 9, 7, 0),
    (3, 13, 11, 128, 136, 1, 1, 1, 0, "s8", "s8", "s8", None, 8, 10, 0),
    (2, 15, 17, 32, 272, 3, 3, 1, 1, "u8", "u8", "s8", "s8", 10, 11, 0),      # second output signed
    (1, 21, 9, 256, 40, 3, 3, 2, 1, "u8", "s8", "u8", None, 12, 9, 4),        # y2 only 4-byte aligned
    (2, 9, 9, 384, 520, 1, 1, 1, 0, "u8", "u8", "u8", "u8", 11, 0, 0),        # second shift 0: pure clip
    (2, 9, 9, 64, 64, 3, 3, 1, 1, "u8", "u8", "u8", None, 6, -2, 0),          # second shift < 0: generic kernel
    (2, 9, 9, 64, 64, 3, 3, 1, 1, "u8", "u8", "u8", "u8", -1, 5, 0),          # first shift < 0
    (2, 10, 7, 5, 9, 3, 3, 1, 1, "s8", "u8", "u8", "s32", 7, 8, 1),           # generic kernel, odd sizes, odd address
    (1, 6, 6, 24, 144, 1, 1, 1, 0, "s8", "u8", "u8", None, 8, 6, 0),          # generic (Cin % 16 != 0)
    (4, 30, 30, 64, 256, 1, 1, 1, 0, "u8", "u8", "u8", "u8", 9, 8, 0),        # several tiles in M and N
]


@pytest.mark.parametrize("variant", [None, 3, 10, 14, 19, 21])
def test_two_output_formats(oracle, variant, forced_variant):
    """One accumulator, two 8-bit outputs with their own fractional lengths and clips: each must be
    the layer evaluated with that format (one rounding each, never a re-rounding of the other)."""
    if variant is not None:
        forced_variant(variant)
    rng = np.random.default_rng(77 + (variant or 0))
    for case in DUAL_CASES:
        B, H, W, Cin, Cout, R, S, st, pd, xt, yt, y2t, rt, sh, sh2, off = case
        if variant in (10,) and R * S * Cin > 64:
            continue
        x, L, res = wl.random_conv_case(rng, B, H, W, Cin, Cout, R, S, st, pd, xt, yt, rt, shift=sh)
        L.fl_y2 = L.fl_x + L.fl_w - sh2
        L.y2_type = y2t
        L.clip_lo2, L.clip_hi2 = (0, int(rng.integers(100, 256))) if y2t == "u8" else (-int(rng.integers(50, 128)), 127)
        want, want2 = oracle.conv2d_fixed_dual(x, L.w, L.bias, L, (st, st), (pd, pd), res)
        xd, wd, bd = (torch.from_numpy(a).to(DEV) for a in (x, L.w, L.bias))
        rd = torch.from_numpy(res).to(DEV) if res is not None else None
        P, Q = L.out_hw
        y = torch.full((B, P, Q, Cout), 77, dtype=f8.TORCH_DTYPE[yt], device=DEV)
        buf = torch.full((B * P * Q * Cout + 64,), 55, dtype=torch.uint8, device=DEV)
        y2 = buf[off:off + B * P * Q * Cout].view(f8.TORCH_DTYPE[y2t]).view(B, P, Q, Cout)
        f8.f8_conv2d_fixed_dual(xd, wd, bd, y, y2, L, (st, st), (pd, pd), rd)
        torch.cuda.synchronize()
        assert_same(y.cpu().numpy(), want, "dual case %s variant %s, first" % (str(case), variant))
        assert_same(y2.cpu().numpy(), want2, "dual case %s variant %s, second" % (str(case), variant))
        assert int(buf[off + B * P * Q * Cout:].min()) == 55 and (off == 0 or int(buf[:off].min()) == 55)


# ------------------------------------------------------------------------- measurement aids

def test_profile_graph_replay_and_copy(oracle):
    """The per-layer profiler leaves the chain's output unchanged; a captured HIP graph of the
    chain reproduces the eager bits on every replay, with eager work between replays; the
    copy yardstick copies."""
    x, net = wl.config4(batch=4, hw=64)
    xt = torch.from_numpy(x).to(DEV)
    chain = f8.Chain(net).prepare(4)
    out = torch.empty((4,) + chain.out_shape, dtype=chain.out_dtype, device=DEV)
    chain.run(xt, out)
    torch.cuda.synchronize()
    eager = out.clone()
    want = oracle.run_network_parallel(net, x, host_threads())
    assert_same(eager.cpu().numpy(), want, "eager")
    ms = chain.profile(xt, out, repeats=2)
    assert len(ms) == len(net.layers) and all(t >= 0 for t in ms) and sum(ms) > 0
    assert torch.equal(out, eager)
    # the stem and the max pool behind it run as one kernel, accounted to the stem
    assert chain.layer_info(0, 4)[0] == "stem_pool_fused" and chain.layer_info(1, 4) == ("(fused)", 0.0, 0.0)
    name, ops, nbytes = chain.layer_info(2, 4)
    assert name and ops > 0 and nbytes > 0
    graph = chain.capture(xt, out)
    for i in range(4):
        out.fill_(i)                                   # eager work between the replays
        scratch = torch.randn(1 << 16, device=DEV).sum()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), "replay %d" % i
    del scratch
    src = torch.randint(0, 256, (1 << 20,), dtype=torch.uint8, device=DEV)
    dst = torch.zeros_like(src)
    f8.f8_copy_bytes(src, dst)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)


def test_chain_channel_padding(oracle):
    """Dense layers whose input channel count is not a multiple of 16 run in the chain on a
    zero-padded copy of input and weights: same bits as the oracle and as the single-layer
    entry point, which takes the generic kernel."""
    rng = np.random.default_rng(4242)
    B, H, W = 3, 13, 11
    x = wl.draw_u8(rng, (B, H, W, 20))
    net = wl.Net(name="odd_channels", in_hw=(H, W), in_c=20, x_type="u8", fl_x=4)
    specs = [(20, 40, 3, 1, 1, "u8", "u8"), (40, 24, 1, 1, 0, "u8", "s8"), (24, 36, 3, 2, 1, "s8", "u8")]
    hw, src = (H, W), 0
    for i, (cin, cout, k, st, pd, xt, yt) in enumerate(specs):
        _, L, _ = wl.random_conv_case(rng, 1, hw[0], hw[1], cin, cout, k, k, st, pd, xt, yt, None)
        L.src, L.dst, L.name = src, src + 1, "l%d" % i
        if i:
            L.fl_x = net.layers[-1].fl_y
            L.fl_y = max(0, L.fl_x + L.fl_w - 6)
        net.layers.append(L)
        hw, src = L.out_hw, src + 1
    net.fl_x = net.layers[0].fl_x
    want = oracle.run_network(net, x, keep_all=True)
    chain = f8.Chain(net, keep_all=True).prepare(B)
    out = chain.run(torch.from_numpy(x).to(DEV))
    torch.cuda.synchronize()
    for L in net.layers[:-1]:
        assert_same(chain.tensor(L.dst).cpu().numpy(), want[L.dst], "padded chain " + L.name)
    assert_same(out.cpu().numpy(), want[net.layers[-1].dst], "padded chain output")
    assert "conv_fast" in chain.layer_info(0, B)[0] and "conv_fast" in chain.layer_info(2, B)[0]
    t = {0: x}
    for L in net.layers:
        t[L.dst] = gpu_layer(L, t[L.src])
        assert_same(t[L.dst], want[L.dst], "single layer " + L.name)


# ------------------------------------------------------------------------- random geometry

def test_random_geometry_fuzz(oracle):
    """Seeded random layer geometries (window, stride, padding, channel counts, types, residual
    kinds, shifts) against the oracle: dense and depthwise, every draw bit-exact."""
    rng = np.random.default_rng(20220205)
    types = ["u8", "s8"]
    for it in range(60):
        depthwise = it % 3 == 2
        R = int(rng.choice([1, 1, 2, 3, 3, 5]))
        S = R if rng.random() < 0.8 else int(rng.choice([1, 2, 3, 4]))
        if depthwise:
            R = S = int(rng.choice([3, 3, 3, 5, 2]))
        stride = int(rng.choice([1, 1, 2, 3]))
        pad = int(rng.integers(0, max(R, S)))
        H = int(rng.integers(max(1, R - 2 * pad), 24))
        W = int(rng.integers(max(1, S - 2 * pad), 24))
        B = int(rng.integers(1, 4))
        Cin = int(rng.choice([1, 3, 4, 8, 12, 16, 24, 32, 48, 64, 80, 96, 128, 144, 192, 256]))
        Cout = Cin if depthwise else int(rng.choice([1, 4, 8, 10, 16, 24, 40, 64, 72, 128, 136, 200, 256, 320]))
        xt = types[int(rng.integers(0, 2))]
        yt = "s32" if (rng.random() < 0.1) else types[int(rng.integers(0, 2))]
        rt = None if rng.random() < 0.5 else ["u8", "s8", "s32"][int(rng.integers(0, 3))]
        shift = None if (yt == "s32" or rng.random() < 0.7) else int(rng.choice([0, -1, -3, 1, 16]))
        x, L, res = wl.random_conv_case(rng, B, H, W, Cin, Cout, R, S, stride, pad, xt, yt, rt, shift=shift,
                                        depthwise=depthwise)
        if L.out_hw[0] < 1 or L.out_hw[1] < 1:
            continue
        fn = oracle.dwconv_fixed if depthwise else oracle.conv2d_fixed
        want = fn(x, L.w, L.bias, L, (stride, stride), (pad, pad), res)
        what = "fuzz %d: dw=%s B%d %dx%d C%d->%d k%dx%d s%d p%d %s->%s res %s shift %s" % (
            it, depthwise, B, H, W, Cin, Cout, R, S, stride, pad, xt, yt, rt, shift)
        assert_same(gpu_layer(L, x, res), want, what)
