"""Algorithm 1 under torch.autograd (forward loop: cache the tuple; backward loop: Dequant, UpSampling + add)
and the mask operators of the appendix on operator compression, on the GPU against the CPU oracle."""
import copy

import numpy as np
import pytest
import torch

import oracle
import paper_2208_04187_amd as pkg

pytestmark = pytest.mark.gpu


def _relu_normal(shape, seed):
    return torch.relu(torch.randn(shape, generator=torch.Generator().manual_seed(seed)))


class oracle_saved_tensors(torch.autograd.graph.saved_tensors_hooks):
    """The same rule of what is cached and with which seed as division_saved_tensors, every map taken to the
    host, through the CPU oracle's compress and decompress, and back: what the backward pass has to see."""

    def __init__(self, B, b, seed, min_elements=1024, c16=False):
        self.maps = 0
        seen = {}

        def pack(t):
            eligible = (t.is_cuda and t.dim() in (3, 4, 5) and t.dtype == torch.float32 and t.is_contiguous()
                        and t.numel() >= min_elements and not isinstance(t, torch.nn.Parameter)
                        and not (t.is_leaf and t.requires_grad))
            if not eligible:
                return t
            key = (t.data_ptr(), t._version, tuple(t.shape))
            if key in seen:
                return seen[key]
            dt = oracle.F32_C16 if c16 else oracle.F32
            shape = tuple(t.shape)
            ms = (shape[0], shape[1], 1, shape[2]) if len(shape) == 3 else shape
            xh = t.detach().cpu().numpy().reshape(ms)
            rebuilt = oracle.decompress(oracle.compress(xh, B, b, seed + self.maps, dt), ms, B, b, dt)
            self.maps += 1
            seen[key] = ("rebuilt", torch.from_numpy(rebuilt.reshape(shape)).to(t.device), t)   # t kept: its address stays taken
            return seen[key]

        def unpack(obj):
            return obj[1] if isinstance(obj, tuple) and obj[0] == "rebuilt" else obj

        super().__init__(pack, unpack)


@pytest.mark.parametrize("c16", [False, True])
def test_saved_tensor_hook_caches_the_map_and_rebuilds_it_in_backward(c16):
    shape, B, b, seed = (4, 6, 28, 28), 8, 2, 91
    odt = oracle.F32_C16 if c16 else oracle.F32
    x = _relu_normal(shape, 7300).to("cuda:0")
    w = torch.nn.Parameter(torch.linspace(0.5, 1.5, x.numel(), device="cuda:0").view(shape))
    h = x.clone().requires_grad_(True)
    hooks = pkg.division_saved_tensors(B, b, seed, c16=c16)
    with hooks:
        y = (h * 1.0) * w            # autograd saves the intermediate map (h * 1.0) for w's gradient
        loss = y.sum()
    loss.backward()
    assert hooks.cached_maps == 1
    assert hooks.cached_bytes == pkg.division_packed_bytes(*shape, B, b, c16=c16)
    # dL/dw is the reconstructed map itself, bit for bit what the oracle rebuilds from the oracle's tuple
    ref = oracle.decompress(oracle.compress(x.cpu().numpy(), B, b, seed, odt), shape, B, b, odt)
    assert np.array_equal(w.grad.cpu().numpy(), ref)
    # dL/dh needs only w, which is a parameter and is never cached
    assert torch.equal(h.grad, w.detach())


@pytest.mark.parametrize("shape", [(3, 8, 200), (2, 4, 6, 20, 12)])
def test_saved_tensor_hook_takes_1d_and_3d_maps(shape):
    B, b, seed = 8, 4, 17
    g = torch.Generator().manual_seed(len(shape))
    x = torch.randn(shape, generator=g).to("cuda:0")
    w = torch.nn.Parameter(torch.full(shape, 2.0, device="cuda:0"))
    h = x.clone().requires_grad_(True)
    hooks = pkg.division_saved_tensors(B, b, seed)
    with hooks:
        loss = ((h * 1.0) * w).sum()
    loss.backward()
    assert hooks.cached_maps == 1
    oshape = shape if len(shape) == 5 else (shape[0], shape[1], 1, shape[2])
    xh = x.cpu().numpy().reshape(oshape)
    ref = oracle.decompress(oracle.compress(xh, B, b, seed), oshape, B, b).reshape(shape)
    assert np.array_equal(w.grad.cpu().numpy(), ref)


def test_a_map_saved_by_two_nodes_is_cached_once():
    shape, B, b, seed = (2, 8, 14, 14), 8, 2, 5
    x = _relu_normal(shape, 11).to("cuda:0")
    w1 = torch.nn.Parameter(torch.full(shape, 2.0, device="cuda:0"))
    w2 = torch.nn.Parameter(torch.full(shape, 3.0, device="cuda:0"))
    h = x.clone().requires_grad_(True)
    hooks = pkg.division_saved_tensors(B, b, seed)
    with hooks:
        m = h * 1.0
        loss = (m * w1).sum() + (m * w2).sum()       # both products save m
    loss.backward()
    assert hooks.cached_maps == 1 and hooks.compress_calls == 1 and hooks.decompress_calls == 1
    ref = oracle.decompress(oracle.compress(x.cpu().numpy(), B, b, seed), shape, B, b)
    assert np.array_equal(w1.grad.cpu().numpy(), ref) and np.array_equal(w2.grad.cpu().numpy(), ref)


@pytest.mark.parametrize("group", [1, 3, 8])
def test_deferred_groups_of_mixed_shapes_match_the_oracle_map_by_map(group):
    B, b, seed = 8, 2, 40
    shapes = [(2, 8, 28, 28), (2, 8, 28, 28), (2, 16, 14, 14), (2, 4, 56, 56), (2, 16, 14, 14), (3, 8, 128), (2, 8, 28, 28)]
    xs = [_relu_normal(s, 100 + i).to("cuda:0") for i, s in enumerate(shapes)]
    ws = [torch.nn.Parameter(torch.full(s, 1.0 + i, device="cuda:0")) for i, s in enumerate(shapes)]
    hs = [x.clone().requires_grad_(True) for x in xs]
    hooks = pkg.division_saved_tensors(B, b, seed, group=group)
    with hooks:
        loss = sum(((h * 1.0) * w).sum() for h, w in zip(hs, ws))
    assert hooks.cached_maps == len(shapes)
    assert hooks.compress_calls == -(-len(shapes) // group)        # whole groups, the rest on leaving the context
    loss.backward()
    assert hooks.decompress_calls == -(-len(shapes) // group)
    for i, (x, w, s) in enumerate(zip(xs, ws, shapes)):
        ms = (s[0], s[1], 1, s[2]) if len(s) == 3 else s
        ref = oracle.decompress(oracle.compress(x.cpu().numpy().reshape(ms), B, b, seed + i), ms, B, b).reshape(s)
        assert np.array_equal(w.grad.cpu().numpy(), ref), i


def test_backward_inside_the_context_compresses_what_still_waits():
    shape, B, b, seed = (2, 8, 28, 28), 8, 2, 3
    x = _relu_normal(shape, 1).to("cuda:0")
    w = torch.nn.Parameter(torch.ones(shape, device="cuda:0"))
    h = x.clone().requires_grad_(True)
    with pkg.division_saved_tensors(B, b, seed, group=8) as hooks:
        loss = ((h * 1.0) * w).sum()
        loss.backward()                                   # the map still waited: it is compressed now, then rebuilt
    ref = oracle.decompress(oracle.compress(x.cpu().numpy(), B, b, seed), shape, B, b)
    assert np.array_equal(w.grad.cpu().numpy(), ref)


def test_mask_operators_have_the_exact_gradients():
    """Relu, Max-Pooling and Dropout keep an exact 1-bit mask: their input gradients are those of the plain
    operators (no quantisation error), also under the hook."""
    g = torch.Generator().manual_seed(3)
    x = torch.randn((4, 8, 28, 28), generator=g).to("cuda:0")
    up = torch.randn((4, 8, 28, 28), generator=g).to("cuda:0")
    a = x.clone().requires_grad_(True)
    with pkg.division_saved_tensors(8, 2, 1) as hooks:
        y = pkg.DivisionReLU()(a)
    y.backward(up)
    assert hooks.cached_maps == 0                              # the operator saved its mask, not a map
    assert torch.equal(y, torch.relu(x)) and torch.equal(a.grad, torch.where(x > 0, up, torch.zeros_like(up)))
    # Max-Pooling, k = 2 (tie-free input): the library's own gradient
    a = x.clone().requires_grad_(True)
    r = x.clone().requires_grad_(True)
    with pkg.division_saved_tensors(8, 2, 1):
        y = pkg.DivisionMaxPool2d(2)(a)
    yr = torch.nn.functional.max_pool2d(r, 2)
    gy = torch.randn(y.shape, generator=g).to("cuda:0")
    y.backward(gy)
    yr.backward(gy)
    assert torch.equal(y, yr) and torch.equal(a.grad, r.grad)
    # Dropout: out = V (.) x, grad = V (.) grad, the same V; no rescaling
    d = pkg.DivisionDropout(0.3, seed=9)
    a = x.clone().requires_grad_(True)
    y = d(a)
    y.backward(up)
    keep = y != 0
    assert torch.equal(y, torch.where(keep, x, torch.zeros_like(x)))
    assert torch.equal(a.grad, torch.where(keep, up, torch.zeros_like(up)))
    assert 0.65 < keep.float().mean().item() < 0.75
    d.eval()
    assert d(x) is x


def _block(seed):
    torch.manual_seed(seed)
    return torch.nn.Sequential(
        torch.nn.Conv2d(3, 8, 3, padding=1, bias=False), torch.nn.BatchNorm2d(8), pkg.DivisionReLU(), pkg.DivisionMaxPool2d(2),
        torch.nn.Conv2d(8, 16, 3, padding=1, bias=False), torch.nn.BatchNorm2d(16), pkg.DivisionReLU(),
        torch.nn.Conv2d(16, 16, 3, padding=1, bias=False), torch.nn.BatchNorm2d(16), pkg.DivisionReLU(),
        torch.nn.Conv2d(16, 4, 1, bias=True)).to("cuda:0")


@pytest.mark.parametrize("group,c16", [(8, False), (1, False), (3, True)])
def test_conv_bn_relu_stack_gets_the_gradients_of_the_oracles_reconstruction(group, c16):
    """A small conv-BN-Relu(-MaxPool) stack trained one step under the hook: every parameter gradient must be
    what the same stack gives when each cached map is replaced by the ORACLE's reconstruction of it (same
    seeds), i.e. Algorithm 1 with the CPU oracle as the codec."""
    B, b, seed = 8, 2, 1234
    net = _block(5)
    ref_net = copy.deepcopy(net)
    x = torch.randn((8, 3, 56, 56), generator=torch.Generator().manual_seed(8)).to("cuda:0")
    target = torch.randn((8, 4, 28, 28), generator=torch.Generator().manual_seed(9)).to("cuda:0")
    hooks = pkg.division_saved_tensors(B, b, seed, group=group, c16=c16)
    with hooks:
        loss = ((net(x) - target) ** 2).mean()
    loss.backward()
    ref_hooks = oracle_saved_tensors(B, b, seed, c16=c16)
    with ref_hooks:
        ref_loss = ((ref_net(x) - target) ** 2).mean()
    ref_loss.backward()
    assert hooks.cached_maps == ref_hooks.maps and hooks.cached_maps >= 8
    assert hooks.compress_calls == -(-hooks.cached_maps // group)
    assert hooks.cached_bytes * 6 < hooks.original_bytes
    assert torch.equal(loss, ref_loss)
    for (n, p), (_, q) in zip(net.named_parameters(), ref_net.named_parameters()):
        assert p.grad is not None and torch.isfinite(p.grad).all(), n
        # the same kernels run on bit-identical inputs; the tolerance only covers a backward kernel that
        # accumulates in an order of its own choosing
        assert torch.allclose(p.grad, q.grad, rtol=1e-5, atol=1e-7), n
    # and the reconstruction matters: without the codec the gradients are different
    plain = copy.deepcopy(ref_net)
    plain.zero_grad()
    ((plain(x) - target) ** 2).mean().backward()
    assert not torch.allclose(next(plain.parameters()).grad, next(net.parameters()).grad, rtol=1e-5, atol=1e-7)
