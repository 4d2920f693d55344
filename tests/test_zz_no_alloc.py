"""ng_step_static -- the step for callers that cannot allocate: its kernels' scratch lies in a device
array of the library instead of the caller's workspace.  Checked through the C ABI against ng_step
on a twin layer set fed the same bytes: same kernels in the same order, so every state buffer and
every weight must agree bit for bit.  Two calls in a row share the one array, the second on a
smaller layer set (stale contents of the first must not matter), then the two interleaved."""
import pytest
import torch

from paper_2410_16029_amd import binding as B
from paper_2410_16029_amd import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


class Twin:
    """Two layer sets over the same shapes and hyper-parameters, refreshed from the same gradient."""

    def __init__(self, shapes, r, s, dtype, seed, k=16, **kw):
        self.shapes = shapes
        self.stream = workloads.TorchGradientStream(shapes, k, 0.01, seed, dtype, DEV)
        self.Wa = workloads.torch_weights(shapes, seed, dtype, DEV)
        self.Wb = [w.clone() for w in self.Wa]
        self.a = B.LayerSet(shapes, r, s=s, dtype=dtype, device=DEV, **kw)   # ng_step_static
        self.b = B.LayerSet(shapes, r, s=s, dtype=dtype, device=DEV, **kw)   # ng_step
        G = self.stream.next_set()
        self.a.refresh(G)
        self.b.refresh(G)
        self.G = G

    def step(self, lr=1e-3, fresh=True):
        if fresh:
            self.G = self.stream.next_set()
        self.a.step_static(self.G, self.Wa, lr)
        self.b.step(self.G, self.Wb, lr)

    def assert_equal(self, label):
        torch.cuda.synchronize()
        assert self.a.status() == B.NG_OK and self.b.status() == B.NG_OK
        for i in range(len(self.shapes)):
            assert self.a.counters(i) == self.b.counters(i), (label, i)
            assert torch.equal(self.Wa[i], self.Wb[i]), (label, "W", i)
            assert torch.equal(self.a.P(i), self.b.P(i)), (label, "P", i)
            # M, V, the ring, the Gram block with w, N: the whole buffers (init cleared them, padding included)
            for buf in (B.NG_BUF_M, B.NG_BUF_V, B.NG_BUF_H, B.NG_BUF_K, B.NG_BUF_N):
                assert torch.equal(self.a.buffers[i][buf], self.b.buffers[i][buf]), (label, "buffer", buf, i)
        # and the weights did move
        assert not torch.equal(self.Wa[0], workloads.torch_weights(self.shapes[:1], self.seed0, self.dtype0, DEV)[0])


def _twin(shapes, r, s, dtype, seed, **kw):
    t = Twin(shapes, r, s, dtype, seed, **kw)
    t.seed0, t.dtype0 = seed, dtype
    return t


def test_static_scratch_step_matches_workspace_step_on_two_calls_in_a_row():
    # first the larger input: bf16, ragged shapes (padded gradient tails, Gram-row partials) ...
    big = _twin([(384, 520), (200, 333), (520, 384), (130, 75)], 64, 4, "bf16", seed=101)
    for _ in range(3):
        big.step()
    big.assert_equal("bf16 set")
    # ... then, on the same array, a smaller one of another kind: fp32, ranks <= 16 (the row-chunk
    # sums of the small-rank projection live in the scratch as well), fewer and smaller matrices
    small = _twin([(129, 66), (64, 130)], [5, 8], 3, "f32", seed=103, k=12)
    for _ in range(4):
        small.step()
    small.assert_equal("small fp32 set")
    # interleaved on one stream: each call rewrites all it reads
    for _ in range(2):
        big.step()
        small.step()
    big.assert_equal("bf16 set, interleaved")
    small.assert_equal("small fp32 set, interleaved")
    # fp32 MFMA path and s = 0
    mid = _twin([(150, 203)], 24, 0, "f32", seed=105, k=8)
    mid.step()
    mid.step()
    mid.assert_equal("fp32, s = 0")
    # right-side matrices, bf16 history slots, the low-memory projector, phase events recorded
    opt = _twin([(333, 200), (200, 333)], 24, 3, "bf16", seed=109, k=24, sides="auto", hist_dtype="bf16",
                proj_dtype="bf16")
    B.ng_set_profiling(opt.a.st, True)
    for _ in range(4):
        opt.step()
    opt.assert_equal("bf16 options")
    ms, steps = B.ng_get_phase_ms(opt.a.st)
    assert steps == 4 and all(x >= 0.0 for x in ms)


def test_static_scratch_rejects_layer_sets_beyond_its_size():
    # 300 matrices x 64 slots: 128 KiB of reduction partials each, 37.5 MiB in all, above the 32 MiB array
    shapes = [(64, 96)] * 300
    ls = B.LayerSet(shapes, 24, s=64, dtype="f32", device=DEV)
    G = workloads.TorchGradientStream(shapes, 8, 0.01, 107, "f32", DEV).next_set()
    W = workloads.torch_weights(shapes, 107, "f32", DEV)
    ls.refresh(G)
    before = [w.clone() for w in W[:3]]
    with pytest.raises(B.NgError) as e:
        ls.step_static(G, W, 1e-3)
    assert e.value.code == B.NG_ERR_WORKSPACE
    assert ls.counters(0) == (0, 0, 0, 1)          # nothing ran, nothing counted
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(before, W[:3]))
    ls.step(G, W, 1e-3)                            # the workspace-backed step takes the same set
    assert ls.status() == B.NG_OK and ls.counters(0) == (1, 1, 1, 1)
