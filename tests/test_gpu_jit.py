"""Just-in-time layer decode (ecf8_jit_*, paper Section 3.3) on the GPU: every layer's weights, as
the consumer stream sees them after acquire(), equal the original tensors; buffers are reused
only after release(); misuse is reported, not executed."""
import numpy as np
import pytest
import torch

from paper_2510_02676_amd import ecf8, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _rand_bytes(n, seed, conc=0.4):
    rng = np.random.default_rng(seed)
    p = rng.dirichlet(np.ones(16) * conc)
    e = rng.choice(16, size=n, p=p).astype(np.uint8)
    return ((rng.integers(0, 2, n, dtype=np.uint8) << 7) | (e << 3) | rng.integers(0, 8, n, dtype=np.uint8)).astype(np.uint8)


def _layers(n_layers, shapes, seed=0, **enc):
    """n_layers layers of len(shapes) tensors each; returns (originals on the device, [(hdrs, d_blobs)])."""
    orig, packed = [], []
    for l in range(n_layers):
        ws, hdrs, blobs = [], [], []
        for i, (r, c) in enumerate(shapes):
            x = _rand_bytes(r * c, seed + 100 * l + i, conc=0.25 + 0.05 * ((l + i) % 5))
            b = ecf8.ecf8_encode(x, r, c, **enc)
            ws.append(torch.from_numpy(x.reshape(r, c)).to(DEV))
            hdrs.append(b.header)
            blobs.append(b.to(DEV))
        orig.append(ws)
        packed.append((hdrs, blobs))
    return orig, packed


@pytest.mark.parametrize("n_buffers", [1, 2, 3])
def test_forward_passes_see_exact_weights(orc, n_buffers):
    shapes = [(256, 1024), (1024, 256), (97, 515), (1, 7), (640, 1024)]
    orig, packed = _layers(6, shapes)
    # one tensor also against the oracle's own decode of the product's blob
    dec, _ = orc.container_decode(packed[3][1][2].cpu().numpy())
    assert np.array_equal(dec, orig[3][2].cpu().numpy().reshape(-1))
    jit = ecf8.Jit(packed, n_buffers=n_buffers)
    compute = torch.cuda.Stream()
    results = []
    for _ in range(2):                                   # two forward passes over the stack
        jit.prefetch(0)
        for l in range(6):
            if n_buffers > 1 and l + 1 < 6:
                jit.prefetch(l + 1)                      # overlaps this layer's "compute"
            ws = jit.acquire(l, compute)
            with torch.cuda.stream(compute):
                results.append([(a == b).all() for a, b in zip(ws, orig[l])])
            jit.release(l, compute)
            if n_buffers == 1 and l + 1 < 6:
                jit.prefetch(l + 1)
    torch.cuda.synchronize()
    assert all(bool(t) for layer in results for t in layer)
    jit.close()


def test_buffer_is_not_overwritten_before_release(orc):
    """The consumer keeps a layer busy for a long time; the decode of the layer that reuses the
    buffer is queued meanwhile and must wait for the release point."""
    shapes = [(1024, 1024), (512, 2048)]
    orig, packed = _layers(4, shapes, seed=7)
    jit = ecf8.Jit(packed, n_buffers=2)
    compute = torch.cuda.Stream()
    big = torch.randn(4096, 4096, device=DEV)
    checks = []
    jit.prefetch(0)
    jit.prefetch(1)
    for l in range(4):
        ws = jit.acquire(l, compute)
        with torch.cuda.stream(compute):
            acc = big
            for _ in range(6):                           # a few ms of unrelated work first
                acc = acc @ big
            checks.append([(a == b).all() for a, b in zip(ws, orig[l])])
        jit.release(l, compute)
        if l + 2 < 4:
            jit.prefetch(l + 2)                          # same buffer as layer l, queued at once
    torch.cuda.synchronize()
    assert all(bool(t) for layer in checks for t in layer)
    jit.close()


@pytest.mark.parametrize("cap", [1, 7, 64, 100000])
def test_decode_workgroup_cap(orc, cap):
    """A cap on the decode launches' workgroups changes who decodes what, never the bytes."""
    orig, packed = _layers(2, [(512, 1024), (300, 700), (2048, 1024)], seed=11)
    jit = ecf8.Jit(packed, n_buffers=2)
    jit.set_decode_workgroups(cap)
    s = torch.cuda.current_stream()
    for l in range(2):
        jit.prefetch(l)
        assert all(torch.equal(a, b) for a, b in zip(jit.acquire(l, s), orig[l]))
        jit.release(l, s)
    torch.cuda.synchronize()
    jit.close()
    x = _rand_bytes(3_000_001, 5)
    b = ecf8.ecf8_encode(x, 1, x.size)
    out = torch.full((x.size,), 0xEE, dtype=torch.uint8, device=DEV)
    batch = ecf8.Batch([b.header], [b.to(DEV)], [out])
    batch.info.max_workgroups = cap
    ecf8.ecf8_decode_batched(batch)
    torch.cuda.synchronize()
    exp, _, _ = orc.roundtrip(x)
    assert np.array_equal(out.cpu().numpy(), exp)


def test_misuse_is_reported():
    orig, packed = _layers(3, [(64, 64)], seed=3)
    jit = ecf8.Jit(packed, n_buffers=2)
    s = torch.cuda.current_stream()
    with pytest.raises(ecf8.Ecf8Error) as e:
        jit.acquire(0, s)                                # nothing prefetched
    assert e.value.code == ecf8.E_ARG
    jit.prefetch(0)
    with pytest.raises(ecf8.Ecf8Error):
        jit.prefetch(2)                                  # buffer 0 holds layer 0
    with pytest.raises(ecf8.Ecf8Error):
        jit.release(0, s)                                # not acquired yet
    with pytest.raises(ecf8.Ecf8Error):
        jit.acquire(2, s)                                # buffer 0 is ready for layer 0, not 2
    with pytest.raises(ecf8.Ecf8Error):
        jit.prefetch(3)                                  # no such layer
    ws = jit.acquire(0, s)
    assert torch.equal(ws[0], orig[0][0])
    with pytest.raises(ecf8.Ecf8Error):
        jit.prefetch(2)                                  # still acquired
    jit.release(0, s)
    jit.prefetch(2)
    assert torch.equal(jit.acquire(2, s)[0], orig[2][0])
    jit.release(2, s)
    torch.cuda.synchronize()
    jit.close()
    with pytest.raises(ecf8.Ecf8Error) as e:
        ecf8.Jit(packed, n_buffers=2, buffer_bytes=1024)  # a 64x64 layer does not fit 1 KiB
    assert e.value.code == ecf8.E_CAPACITY


def test_layers_of_wider_formats_and_mixed_managers():
    """A manager whose layers alternate between FP8 (ecf8 container) and BF16 / E5M2 (wide container): what the
    consumer sees after acquire equals the original tensors, over two passes with two buffers."""
    from paper_2510_02676_amd import ecfw
    shapes = [(256, 512), (128, 1024), (64, 256)]
    layers, originals = [], []
    for l in range(6):
        kind = l % 3
        hdrs, blobs, orig = [], [], []
        for j, (r, c) in enumerate(shapes):
            if kind == 0:
                w = synth.make_weight(r, c, 1.8, 0.02, 50 + l, tensor_id=j)
                b = ecf8.ecf8_encode(w.numpy(), r, c)
            elif kind == 1:
                w = synth.make_bf16(r, c, 1.8, 0.02, 50 + l, tensor_id=j)
                b = ecfw.ecfw_encode(ecfw.FMT_BF16, w, r, c)
                w = w.view(torch.bfloat16)
            else:
                w = synth.make_e5m2(r, c, 1.8, 0.02, 50 + l, tensor_id=j)
                b = ecfw.ecfw_encode(ecfw.FMT_E5M2, w, r, c)
            hdrs.append(b.header)
            blobs.append(b.to(DEV))
            orig.append(w.to(DEV))
        layers.append((hdrs, blobs))
        originals.append(orig)
    jit = ecf8.Jit(layers, n_buffers=2)
    s = torch.cuda.current_stream()
    for _ in range(2):
        jit.prefetch(0)
        for l in range(6):
            if l + 1 < 6:
                jit.prefetch(l + 1)
            views = jit.acquire(l, s)
            for v, o in zip(views, originals[l]):
                assert v.dtype == o.dtype and torch.equal(v.view(torch.uint8), o.view(torch.uint8))
            jit.release(l, s)
    torch.cuda.synchronize()
    jit.close()


def test_decode_launches_replay_from_a_hip_graph():
    """The decode calls allocate nothing, synchronise nothing and clear nothing with memsets, so a caller may
    capture them into a HIP graph: four per-layer FP8 launches and one BF16 launch are captured once and
    replayed three times, with the outputs poisoned and eager work in between; every replay must reproduce
    the eager result."""
    from paper_2510_02676_amd import ecfw
    orig, packed = _layers(4, [(256, 1024), (64, 4096), (512, 512)], seed=9)
    batches, outs = [], []
    for hdrs, blobs in packed:
        o = [torch.empty((h.rows, h.cols), dtype=torch.uint8, device=DEV) for h in hdrs]
        batches.append(ecf8.Batch(hdrs, blobs, o))
        outs.append(o)
    wb = synth.make_bf16(300, 700, 1.8, 0.02, 4)
    wblob = ecfw.ecfw_encode(ecfw.FMT_BF16, wb, 300, 700)
    d_wblob, wout = wblob.to(DEV), torch.empty(300 * 700, dtype=torch.bfloat16, device=DEV)
    d_wb = wb.view(torch.bfloat16).reshape(-1).to(DEV)

    def poison():
        for o in outs:
            for t in o:
                t.fill_(0xEE)
        wout.view(torch.int16).fill_(0x1111)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):            # warm-up outside the capture, as graph capture asks for
        for b in batches:
            ecf8.ecf8_decode_batched(b, side)
        ecfw.ecfw_decode(d_wblob, wblob.header, wout, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        s = torch.cuda.current_stream()
        for b in batches:
            ecf8.ecf8_decode_batched(b, s)
        ecfw.ecfw_decode(d_wblob, wblob.header, wout, stream=s)
    for _ in range(3):
        poison()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for o, ws in zip(outs, orig):
            for t, w in zip(o, ws):
                assert torch.equal(t, w)
        assert torch.equal(wout.view(torch.int16), d_wb.view(torch.int16))
        # eager work between replays
        poison()
        ecf8.ecf8_decode_batched(batches[0])
        torch.cuda.synchronize()
        assert all(torch.equal(t, w) for t, w in zip(outs[0], orig[0]))


def test_forward_hooks_decode_just_in_time():
    """Section 3.3 as the paper states it: per-layer decode from PyTorch forward hooks.  A stack of synthetic
    layers (two FP8 matrices each, multiplied by this library's GEMM on uncompressed weights) holds no weights
    of its own; JitHooks decodes each layer right before its forward pass into one of two shared buffers and
    queues the next layer's decode.  Outputs equal those of the same stack on resident weights bit for bit,
    over three passes, and outside a layer's forward pass its weight attributes are empty."""
    from paper_2510_02676_amd.jit_hooks import JitHooks

    class Layer(torch.nn.Module):
        def __init__(self, up=None, down=None):
            super().__init__()
            self.up, self.down = up, down

        def forward(self, x):                      # x: (M, 1024) E4M3 bytes
            assert self.up.numel() and self.down.numel()
            h = ecf8.ecf8_gemm_fp8_raw(self.up, x)                               # (M, 512) fp32
            hq = (h / h.abs().amax(dim=1, keepdim=True).clamp(min=1e-30) * 448.0).to(torch.float8_e4m3fn).view(torch.uint8)
            y = ecf8.ecf8_gemm_fp8_raw(self.down, hq.contiguous())               # (M, 1024) fp32
            return (y / y.abs().amax(dim=1, keepdim=True).clamp(min=1e-30) * 448.0).to(torch.float8_e4m3fn).view(torch.uint8).contiguous()

    L, M = 5, 8
    orig, packed = _layers(L, [(512, 1024), (1024, 512)], seed=77)
    resident = torch.nn.Sequential(*[Layer(*ws) for ws in orig])
    lazy = torch.nn.Sequential(*[Layer() for _ in range(L)])
    jit = ecf8.Jit(packed, n_buffers=2)
    hooks = JitHooks(list(lazy), [["up", "down"]] * L, jit)
    for rep in range(3):
        x = synth.activations(M, 1024, seed=900 + rep).to(DEV)
        want = resident(x)
        got = lazy(x)
        torch.cuda.synchronize()
        assert torch.equal(got, want), rep
        assert all(layer.up.numel() == 0 and layer.down.numel() == 0 for layer in lazy)
    hooks.remove()
    jit.close()
