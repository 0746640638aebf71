"""GPU parity: MobileNet-v1 layer by layer and end to end against the CPU oracle."""
import numpy as np
import pytest

import oracle
from oracle import ACT_RELU6, PAD_SAME
from paper_1901_05350_amd import inputs
from util import assert_close, dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def net():
    data = inputs.mobilenet_v1(seed=4, batch=1)
    probs, logits, acts = oracle.mobilenet_v1_forward(data["image"], data["weights"], return_activations=True)
    return data, probs, logits, acts


def test_layer_by_layer_each_fed_the_oracle_input(net):
    import paper_1901_05350_amd as tfx
    data, probs, logits, acts = net
    w = data["weights"]
    got = host(tfx.tfx_conv2d(dev(data["image"]), dev(w["conv0_w"]), dev(w["conv0_b"]), 2, PAD_SAME, ACT_RELU6))
    assert_close(got, acts[0], "conv0")
    for i in range(13):
        s = oracle.MOBILENET_V1_STRIDES[i]
        got = host(tfx.tfx_depthwise_conv2d(dev(acts[2 * i]), dev(w["dw_w"][i]), dev(w["dw_b"][i]), s, PAD_SAME, ACT_RELU6))
        assert_close(got, acts[2 * i + 1], "dw%d" % (i + 1))
        got = host(tfx.tfx_conv2d(dev(acts[2 * i + 1]), dev(w["pw_w"][i]), dev(w["pw_b"][i]), 1, PAD_SAME, ACT_RELU6))
        assert_close(got, acts[2 * i + 2], "pw%d" % (i + 1))


def test_end_to_end_logits_and_probs(net):
    import torch
    import paper_1901_05350_amd as tfx
    data, probs, logits, acts = net
    model = tfx.MobileNetV1(data["weights"], batch=1)
    p, l = model.forward(dev(data["image"]))
    p, l = host(p), host(l)
    assert_close(l, logits, "logits")
    assert_close(p, probs, "probs")
    assert abs(float(p.astype(np.float64).sum()) - 1.0) < 1e-5
    assert int(p.argmax()) == int(probs.argmax())
    # a second call reuses the workspace and gives the same bits
    p2, l2 = model.forward(dev(data["image"]))
    assert np.array_equal(host(p2), p) and np.array_equal(host(l2), l)
    # logits pointer is optional
    out = torch.empty((1, 1000), dtype=torch.float32, device="cuda:0")
    tfx.tfx_mobilenet_v1_forward(dev(data["image"]), model.struct, model.workspace, out, None)
    assert np.array_equal(host(out), p)


def test_end_to_end_batch_3():
    import paper_1901_05350_amd as tfx
    data = inputs.mobilenet_v1(seed=7, batch=3)
    probs, logits = oracle.mobilenet_v1_forward(data["image"], data["weights"])
    model = tfx.MobileNetV1(data["weights"], batch=3)
    p, l = model.forward(dev(data["image"]))
    assert_close(host(l), logits, "logits batch 3")
    assert_close(host(p), probs, "probs batch 3")


@pytest.mark.parametrize("batch", [8, 64])
def test_end_to_end_benchmark_batches_every_image(batch):
    """The batched forward passes the benchmark times (other tile shapes and kernels than batch 1: filter-stationary
    pointwise kernel, 128 x 128 tiles, several depthwise rows per lane).  Every image of the batch is compared with
    the oracle's forward pass of the whole batch."""
    import paper_1901_05350_amd as tfx
    data = inputs.mobilenet_v1(seed=9, batch=batch)
    model = tfx.MobileNetV1(data["weights"], batch=batch)
    p, l = model.forward(dev(data["image"]))
    p, l = host(p), host(l)
    assert np.isfinite(p).all() and np.isfinite(l).all()
    np.testing.assert_allclose(p.astype(np.float64).sum(axis=1), 1.0, atol=1e-5)
    probs, logits = oracle.mobilenet_v1_forward(data["image"], data["weights"])
    assert_close(l, logits, "logits batch %d" % batch)
    assert_close(p, probs, "probs batch %d" % batch)
    assert np.array_equal(p.argmax(axis=1), probs.argmax(axis=1))


@pytest.mark.parametrize("size,q,classes,batch", [(128, 1, 10, 2), (160, 2, 1000, 1), (192, 3, 1000, 1), (224, 4, 37, 1),
                                                  (100, 2, 5, 3), (256, 1, 1024, 1)])
def test_family_variants_end_to_end(size, q, classes, batch):
    """Width / resolution members of the family (and odd sizes) through tfx_mobilenet_v1_variant_forward."""
    import paper_1901_05350_amd as tfx
    data = inputs.mobilenet_v1(seed=20 + q, batch=batch, image_size=size, width_quarters=q, classes=classes)
    probs, logits = oracle.mobilenet_v1_forward(data["image"], data["weights"])
    model = tfx.MobileNetV1(data["weights"], batch=batch, image_size=size, width_quarters=q)
    assert not model.is_base
    p, l = model.forward(dev(data["image"]))
    p, l = host(p), host(l)
    assert p.shape == (batch, classes)
    assert_close(l, logits, "logits %d/%d" % (q, size))
    assert_close(p, probs, "probs %d/%d" % (q, size))
    np.testing.assert_allclose(p.astype(np.float64).sum(axis=1), 1.0, atol=1e-5)


def test_internal_activations_of_every_block(net):
    """tfx_mobilenet_v1_variant_features against the oracle's activation after each block's pointwise layer; at
    batch 1 blocks 1 - 4 are the fused stem / depthwise / pointwise kernels, so this is their parity test too."""
    import torch
    import paper_1901_05350_amd as tfx
    data, probs, logits, acts = net
    model = tfx.MobileNetV1(data["weights"], batch=1)
    img = dev(data["image"])
    for k in range(1, 14):
        want = acts[2 * k]
        got = model.features(img, k)
        assert tuple(got.shape) == want.shape
        assert_close(host(got), want, "features after block %d" % k)
    # into a caller's buffer, twice: same bits; the forward pass afterwards is unaffected
    out = torch.full(acts[8].shape, -1.0, dtype=torch.float32, device="cuda:0")
    model.features(img, 4, out=out)
    first = host(out).copy()
    model.features(img, 4, out=out)
    assert np.array_equal(host(out), first)
    assert_close(first, acts[8], "features after block 4")
    p, l = model.forward(img)
    assert_close(host(l), logits, "logits after features calls")
    with pytest.raises(tfx.TfxError):
        model.features(img, 14, out=out)
    with pytest.raises(TypeError):
        model.features(img, 6, out=out)   # wrong shape for block 6


@pytest.mark.parametrize("size,q,batch,blocks", [(100, 4, 1, (1, 2, 3, 4, 5, 7, 13)), (100, 2, 3, (1, 6, 13)),
                                                 (160, 4, 2, (1, 4, 12)), (32, 4, 1, (1, 2, 3, 4, 5, 13)),
                                                 (72, 4, 3, (1, 2, 3, 4, 5, 13)), (64, 4, 4, (1, 4))])
def test_internal_activations_of_variants_and_batches(size, q, batch, blocks):
    """Odd map sizes (ragged 4 x 4 patches of the fused kernels, which serve batch 1 to 3), other widths, and batches
    on both sides of that limit."""
    import paper_1901_05350_amd as tfx
    data = inputs.mobilenet_v1(seed=40 + q, batch=batch, image_size=size, width_quarters=q, classes=10)
    probs, logits, acts = oracle.mobilenet_v1_forward(data["image"], data["weights"], return_activations=True)
    model = tfx.MobileNetV1(data["weights"], batch=batch, image_size=size, width_quarters=q)
    img = dev(data["image"])
    for k in blocks:
        got = model.features(img, k)
        assert tuple(got.shape) == acts[2 * k].shape
        assert_close(host(got), acts[2 * k], "features %d/%d block %d" % (q, size, k))


@pytest.mark.parametrize("size,batch,blocks", [(224, 5, (1, 2, 3, 4)), (224, 12, (2, 3)), (200, 16, (1, 2, 3)), (224, 44, (4, 5))])
def test_internal_activations_at_large_batch(size, batch, blocks):
    """From 8192 output pixels on, blocks 1, 2 and 3 of the full-width network run as one filter-stationary launch
    each (the depthwise result computed into the pointwise layer's MFMA operand from a window in LDS); the later
    blocks take the single-op kernels.  200 x 200 images give 100 x 100 and 50 x 50 maps: ragged last patches and
    an odd padding under stride 2."""
    import paper_1901_05350_amd as tfx
    data = inputs.mobilenet_v1(seed=47, batch=batch, image_size=size, width_quarters=4, classes=10)
    probs, logits, acts = oracle.mobilenet_v1_forward(data["image"], data["weights"], return_activations=True)
    model = tfx.MobileNetV1(data["weights"], batch=batch, image_size=size, width_quarters=4)
    img = dev(data["image"])
    for k in blocks:
        got = model.features(img, k)
        assert tuple(got.shape) == acts[2 * k].shape
        assert_close(host(got), acts[2 * k], "features batch %d size %d block %d" % (batch, size, k))
    p, l = model.forward(img)
    assert_close(host(l), logits, "logits batch %d size %d" % (batch, size))


def test_nan_and_inf_through_the_fused_blocks_at_large_batch():
    """A NaN in one image reaches exactly the outputs whose windows hold it, block after block, and no other image;
    +inf and -inf clamp as the oracle's relu6 does (the fused kernels clamp with a median of three and must notice
    the NaN on the side)."""
    import paper_1901_05350_amd as tfx
    batch = 5
    data = inputs.mobilenet_v1(seed=48, batch=batch, image_size=224, width_quarters=4, classes=10)
    img = data["image"].copy()
    img[3, 100, 37, 1] = np.nan
    img[1, 5, 7, 0] = np.inf
    img[4, 200, 220, 2] = -np.inf
    probs, logits, acts = oracle.mobilenet_v1_forward(img, data["weights"], return_activations=True)
    model = tfx.MobileNetV1(data["weights"], batch=batch, image_size=224, width_quarters=4)
    for k in (1, 2, 3):
        got, ref = host(model.features(dev(img), k)), acts[2 * k]
        assert np.isnan(ref).any() and not np.isnan(ref[3]).all() and not np.isnan(ref[[0, 1, 2, 4]]).any()
        assert np.array_equal(np.isnan(got), np.isnan(ref)), "NaN positions after block %d" % k
        ok = ~np.isnan(ref)
        assert_close(got[ok], ref[ok], "finite values after block %d" % k)


def test_base_variant_is_the_plain_entry_point(net):
    import torch
    import paper_1901_05350_amd as tfx
    data, probs, logits, acts = net
    model = tfx.MobileNetV1(data["weights"], batch=1)
    p, _ = model.forward(dev(data["image"]))
    p = host(p).copy()
    out = torch.empty((1, 1000), dtype=torch.float32, device="cuda:0")
    tfx.tfx_mobilenet_v1_variant_forward(tfx.TfxVariant(224, 4, 1000), dev(data["image"]), model.struct, model.workspace, out)
    assert np.array_equal(host(out), p)


def test_workspace_checks(net):
    import torch
    import paper_1901_05350_amd as tfx
    data, *_ = net
    model = tfx.MobileNetV1(data["weights"], batch=1)
    small = torch.empty(1024, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(tfx.TfxError) as e:
        tfx.tfx_mobilenet_v1_forward(dev(data["image"]), model.struct, small, model.probs, None)
    assert e.value.status == -5


def test_forward_captured_in_a_graph_replays_identically(net):
    # the library only enqueues kernels (no allocation, no memset, no host sync), so a forward pass can be
    # captured into a HIP graph; every replay, with eager work in between, must give the eager bits
    import torch
    import paper_1901_05350_amd as tfx
    data, probs, logits, acts = net
    model = tfx.MobileNetV1(data["weights"], batch=1)
    image = dev(data["image"])
    p_eager = host(model.forward(image)[0]).copy()
    l_eager = host(model.logits).copy()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        model.forward(image)
    other = dev(np.random.Generator(np.random.PCG64(99)).uniform(-1, 1, (1, 224, 224, 3)))
    for _ in range(3):
        model.probs.zero_()
        model.logits.zero_()
        # eager work on the same workspace between replays: a different image overwrites every buffer
        model2_out = host(model.forward(other)[0]).copy()
        assert not np.array_equal(model2_out, p_eager)
        g.replay()
        assert np.array_equal(host(model.probs), p_eager)
        assert np.array_equal(host(model.logits), l_eager)


def test_batched_forward_first_called_under_graph_capture():
    """Batch 8 uses kernels batch 1 does not (filter-stationary pointwise kernels, which look up their residency and
    set an LDS attribute on first use).  Here their first call in the process may happen while a graph is being
    captured: the capture must succeed and the replay must match an eager run of the same model."""
    import torch
    import paper_1901_05350_amd as tfx
    data = inputs.mobilenet_v1(seed=11, batch=8, image_size=192, width_quarters=4)   # a size no other test uses at batch 8
    model = tfx.MobileNetV1(data["weights"], batch=8, image_size=192, width_quarters=4)
    image = dev(data["image"])
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        model.forward(image)
    g.replay()
    p_graph = host(model.probs).copy()
    l_graph = host(model.logits).copy()
    model.probs.zero_()
    model.logits.zero_()
    p_eager = host(model.forward(image)[0]).copy()
    assert np.array_equal(p_graph, p_eager) and np.array_equal(l_graph, host(model.logits))
    probs, logits = oracle.mobilenet_v1_forward(data["image"], data["weights"])
    assert_close(l_graph, logits, "logits batch 8 (192 x 192)")


@pytest.mark.parametrize("batch", [33, 61])
def test_forward_in_two_halves_from_batch_32(batch):
    """From batch 32 on the forward pass is two parts of the batch (17 + 16 images), from batch 60 on three (21 + 20 +
    20), all but the first on streams of the library's own, forked from and joined to the caller's.  Every image
    against the oracle; the same bits on a second call; and captured into a graph (fork and joins become edges of the
    graph) every replay gives the eager bits."""
    import torch
    import paper_1901_05350_amd as tfx
    data = inputs.mobilenet_v1(seed=12, batch=batch, image_size=96, width_quarters=2, classes=10)
    probs, logits = oracle.mobilenet_v1_forward(data["image"], data["weights"])
    model = tfx.MobileNetV1(data["weights"], batch=batch, image_size=96, width_quarters=2)
    image = dev(data["image"])
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):          # not the default stream: the fork has to follow the caller's stream
        p, l = model.forward(image)
    stream.synchronize()
    p, l = host(p).copy(), host(l).copy()
    assert_close(l, logits, "logits batch %d" % batch)
    assert_close(p, probs, "probs batch %d" % batch)
    p2, l2 = model.forward(image)
    assert np.array_equal(host(p2), p) and np.array_equal(host(l2), l)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        model.forward(image)
    other = dev(np.random.Generator(np.random.PCG64(98)).uniform(-1, 1, (batch, 96, 96, 3)))
    for _ in range(3):
        assert not np.array_equal(host(model.forward(other)[0]), p)     # eager work on the same workspace in between
        model.probs.zero_()
        g.replay()
        assert np.array_equal(host(model.probs), p) and np.array_equal(host(model.logits), l)


def test_two_host_threads_share_the_second_stream():
    """Two host threads, each with a stream and a model of its own, run batch-32 forward passes at the same time: both
    fork to the library's one second stream (its events are re-recorded call after call, under a lock).  All results
    must have the bits of an undisturbed run."""
    import threading
    import torch
    import paper_1901_05350_amd as tfx
    batch = 32
    data = inputs.mobilenet_v1(seed=13, batch=batch, image_size=64, width_quarters=1, classes=16)
    models = [tfx.MobileNetV1(data["weights"], batch=batch, image_size=64, width_quarters=1) for _ in range(2)]
    images = [dev(data["image"]), dev(data["image"][::-1].copy())]
    want = [host(m.forward(x)[0]).copy() for m, x in zip(models, images)]
    assert not np.array_equal(want[0], want[1])
    outs = [[torch.zeros_like(m.probs) for _ in range(20)] for m in models]
    streams = [torch.cuda.Stream() for _ in models]
    torch.cuda.synchronize()

    def worker(i):
        with torch.cuda.stream(streams[i]):
            for o in outs[i]:
                tfx.tfx_mobilenet_v1_variant_forward(models[i].variant, images[i], models[i].struct, models[i].workspace, o)

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    for i in range(2):
        for o in outs[i]:
            assert np.array_equal(host(o), want[i])


# ---- the chained small-map kernel (batch 1, full width: blocks 5 .. 13, pool, fully connected, softmax in one launch) ----
@pytest.mark.parametrize("size,classes", [(32, 3), (64, 1000), (100, 5), (128, 1024), (160, 37), (192, 1000), (250, 130),
                                          (256, 1)])
def test_chained_kernel_other_input_sizes_and_class_counts(size, classes):
    """Full-width members at batch 1 take the chained kernel for every input size: maps from 32 x 32 down to 1 x 1,
    ragged 16-pixel row tiles, both pointwise tile widths, class counts that are not multiples of 4 or 128."""
    import paper_1901_05350_amd as tfx
    data = inputs.mobilenet_v1(seed=50 + size, batch=1, image_size=size, width_quarters=4, classes=classes)
    probs, logits = oracle.mobilenet_v1_forward(data["image"], data["weights"])
    model = tfx.MobileNetV1(data["weights"], batch=1, image_size=size, width_quarters=4)
    p, l = model.forward(dev(data["image"]))
    p, l = host(p).copy(), host(l).copy()
    assert_close(l, logits, "logits 1.0/%d, %d classes" % (size, classes))
    assert_close(p, probs, "probs 1.0/%d, %d classes" % (size, classes))
    # the same bits on every call (the kernel's tasks run in a different order each time)
    for _ in range(5):
        p2, l2 = model.forward(dev(data["image"]))
        assert np.array_equal(host(p2), p) and np.array_equal(host(l2), l)


@pytest.mark.parametrize("size,q,classes", [(128, 1, 1000), (32, 1, 3), (224, 1, 10), (160, 2, 37), (96, 2, 1024),
                                            (192, 3, 1000), (224, 3, 130), (250, 3, 5)])
def test_chained_kernel_other_widths(size, q, classes):
    """The narrower members at batch 1 take the chained kernel from block 5 on: 64 q / 128 q / 256 q channels, i.e. a K
    split over 4 wavefronts for K = 64 and 192, 2 q slices of the fully connected layer; the stem kernel for 8 q
    filters clears the task flags."""
    import paper_1901_05350_amd as tfx
    data = inputs.mobilenet_v1(seed=70 + size + q, batch=1, image_size=size, width_quarters=q, classes=classes)
    probs, logits, acts = oracle.mobilenet_v1_forward(data["image"], data["weights"], return_activations=True)
    model = tfx.MobileNetV1(data["weights"], batch=1, image_size=size, width_quarters=q)
    image = dev(data["image"])
    p, l = model.forward(image)
    p, l = host(p).copy(), host(l).copy()
    assert_close(l, logits, "logits %d/4 width, %d, %d classes" % (q, size, classes))
    assert_close(p, probs, "probs %d/4 width, %d, %d classes" % (q, size, classes))
    for _ in range(5):
        p2, l2 = model.forward(image)
        assert np.array_equal(host(p2), p) and np.array_equal(host(l2), l)
    # the layers in front of the chain, and the same blocks as single kernels
    for k in (4, 5, 13):
        assert_close(host(model.features(image, k)), acts[2 * k], "features %d/4 width, %d, block %d" % (q, size, k))


def test_chained_kernel_of_a_narrow_member_that_gives_up_writes_nan(monkeypatch):
    import paper_1901_05350_amd as tfx
    data = inputs.mobilenet_v1(seed=77, batch=1, image_size=160, width_quarters=2, classes=100)
    probs, logits = oracle.mobilenet_v1_forward(data["image"], data["weights"])
    model = tfx.MobileNetV1(data["weights"], batch=1, image_size=160, width_quarters=2)
    image = dev(data["image"])
    monkeypatch.setenv("TFX_CHAIN_SPIN_LIMIT", "1")
    p, l = model.forward(image)
    assert np.isnan(host(p)).all() and np.isnan(host(l)).all()
    monkeypatch.delenv("TFX_CHAIN_SPIN_LIMIT")
    p, l = model.forward(image)
    assert_close(host(l), logits, "logits after a failed call")
    assert_close(host(p), probs, "probs after a failed call")


def test_chained_kernel_many_calls_back_to_back_give_the_same_bits(net):
    import torch
    import paper_1901_05350_amd as tfx
    data, probs, logits, acts = net
    model = tfx.MobileNetV1(data["weights"], batch=1)
    image = dev(data["image"])
    outs = [(torch.empty_like(model.probs), torch.empty_like(model.logits)) for _ in range(300)]
    for p, l in outs:                      # no synchronisation in between: 300 forward passes queued on the stream
        tfx.tfx_mobilenet_v1_forward(image, model.struct, model.workspace, p, l)
    torch.cuda.synchronize()
    p0, l0 = outs[0][0].cpu().numpy(), outs[0][1].cpu().numpy()
    assert_close(l0, logits, "logits")
    for p, l in outs[1:]:
        assert np.array_equal(p.cpu().numpy(), p0) and np.array_equal(l.cpu().numpy(), l0)


def test_chained_kernel_nan_in_the_image_reaches_every_output(net):
    import paper_1901_05350_amd as tfx
    data, *_ = net
    img = data["image"].copy()
    img[0, 100, 37, 1] = np.nan
    probs, logits = oracle.mobilenet_v1_forward(img, data["weights"])
    assert np.isnan(logits).all() and np.isnan(probs).all()
    model = tfx.MobileNetV1(data["weights"], batch=1)
    p, l = model.forward(dev(img))
    assert np.isnan(host(p)).all() and np.isnan(host(l)).all()


def test_chained_kernel_bounded_waits_give_up_and_report_nan(net, monkeypatch):
    """Every wait inside the chained kernel is bounded.  With the limit forced down to one poll from the host, waits
    give up before their producers are done: the kernel must still run to its end (no hang), flag the failure and
    write NaN to every output instead of numbers computed from unfinished inputs; the next normal call is correct."""
    import paper_1901_05350_amd as tfx
    data, probs, logits, acts = net
    model = tfx.MobileNetV1(data["weights"], batch=1)
    image = dev(data["image"])
    monkeypatch.setenv("TFX_CHAIN_SPIN_LIMIT", "1")
    p, l = model.forward(image)
    assert np.isnan(host(p)).all() and np.isnan(host(l)).all()
    monkeypatch.delenv("TFX_CHAIN_SPIN_LIMIT")
    p, l = model.forward(image)
    assert_close(host(l), logits, "logits after a failed call")
    assert_close(host(p), probs, "probs after a failed call")


def test_chained_blocks_that_give_up_write_nan_not_numbers(net, monkeypatch):
    """Blocks 2 - 4 run as stages of one launch that wait for each other's patches.  With the waits cut to one poll,
    a stage that went ahead without its input must write NaN: every element of block 4's output is then either
    NaN or exactly the value of an undisturbed run, never a number computed from unfinished data."""
    import paper_1901_05350_amd as tfx
    data, probs, logits, acts = net
    model = tfx.MobileNetV1(data["weights"], batch=1)
    image = dev(data["image"])
    for k in (4, 5):   # the staged launch alone, and with block 5's kernel behind it
        good = host(model.features(image, k)).copy()
        assert_close(good, acts[2 * k], "features after block %d" % k)
        monkeypatch.setenv("TFX_CHAIN_SPIN_LIMIT", "1")
        cut = host(model.features(image, k))
        monkeypatch.delenv("TFX_CHAIN_SPIN_LIMIT")
        bad = np.isnan(cut)
        assert bad.any()
        assert np.array_equal(cut[~bad], good[~bad])
        again = host(model.features(image, k))
        assert np.array_equal(again, good)


def test_two_chained_kernels_on_two_streams_at_once(net):
    """Two batch-1 forward passes issued from two host threads on two streams: the chained kernels would compete for
    the CUs (neither grid fully resident, each waiting for workgroups the other keeps out), so the library orders
    them across streams.  All 60 results must have the right bits."""
    import threading
    import torch
    import paper_1901_05350_amd as tfx
    data, probs, logits, acts = net
    models = [tfx.MobileNetV1(data["weights"], batch=1) for _ in range(2)]
    image = dev(data["image"])
    p0 = host(models[0].forward(image)[0]).copy()
    outs = [[torch.zeros_like(m.probs) for _ in range(30)] for m in models]
    streams = [torch.cuda.Stream() for _ in models]
    torch.cuda.synchronize()

    def worker(i):
        with torch.cuda.stream(streams[i]):
            for o in outs[i]:
                tfx.tfx_mobilenet_v1_forward(image, models[i].struct, models[i].workspace, o, None)
    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    for i in range(2):
        for o in outs[i]:
            assert np.array_equal(o.cpu().numpy(), p0)
