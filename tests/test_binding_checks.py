"""The binding refuses query tensors that do not fit the graph before anything is launched (no GPU needed:
the checks run on tensor metadata, and a mismatch must raise before the library is called)."""
import pytest

torch = pytest.importorskip("torch")


class _FakeCuda:
    """Stands in for a GPU tensor: the checks only look at metadata."""

    def __init__(self, shape, dtype, device="cuda:0", contiguous=True):
        self._t = torch.empty(shape, dtype=dtype, device="meta")
        self.shape, self.dtype, self.device = self._t.shape, dtype, torch.device(device)
        self._c = contiguous

    is_cuda = True

    def dim(self):
        return self._t.dim()

    def is_contiguous(self):
        return self._c


@pytest.fixture()
def graph_and_lib(monkeypatch):
    from paper_1912_01059_amd import binding

    def boom():
        raise AssertionError("the library must not be reached")
    monkeypatch.setattr(binding, "lib", boom)
    monkeypatch.setattr(torch, "Tensor", (torch.Tensor, _FakeCuda))  # isinstance checks accept the stand-in
    g = binding.Graph.__new__(binding.Graph)
    g.h, g.N, g.D, g.K, g.L, g.dtype, g.metric = None, 1000, 128, 24, 3, binding.F32, binding.L2
    return binding, g


def test_query_refuses_tensors_that_do_not_fit_the_graph(graph_and_lib):
    binding, g = graph_and_lib
    ok_q = _FakeCuda((10, 128), torch.float32)
    with pytest.raises(TypeError):   # uint8 queries on a float32 graph: the kernel would read 4x past the end
        binding.query(g, _FakeCuda((10, 128), torch.uint8), 10, 10, 0.3)
    with pytest.raises(binding.GgnnError):  # wrong D
        binding.query(g, _FakeCuda((10, 96), torch.float32), 10, 10, 0.3)
    with pytest.raises(binding.GgnnError):  # not 2-D
        binding.query(g, _FakeCuda((1280,), torch.float32), 10, 10, 0.3)
    with pytest.raises(binding.GgnnError):  # not contiguous
        binding.query(g, _FakeCuda((10, 128), torch.float32, contiguous=False), 10, 10, 0.3)
    with pytest.raises(TypeError):   # a host tensor
        binding.query(g, torch.zeros((10, 128)), 10, 10, 0.3)
    good_ids, good_d = _FakeCuda((10, 10), torch.int32), _FakeCuda((10, 10), torch.float32)
    for bad in [(_FakeCuda((10, 10), torch.int64), good_d), (good_ids, _FakeCuda((10, 10), torch.float64)),
                (_FakeCuda((9, 10), torch.int32), good_d), (good_ids, _FakeCuda((10, 5), torch.float32)),
                (_FakeCuda((10, 10), torch.int32, device="cuda:1"), good_d)]:
        with pytest.raises(binding.GgnnError):
            binding.query(g, ok_q, 10, 10, 0.3, out=bad)
    with pytest.raises(binding.GgnnError):  # start points must be int32 on the same device
        binding.query(g, ok_q, 10, 10, 0.3, start_ids=_FakeCuda((4,), torch.int64))
    with pytest.raises(binding.GgnnError):
        binding.query_static(g, ok_q, 10, 10, 0.3, (good_ids, good_d), counters=_FakeCuda((10, 2), torch.int32))
    # a uint8 graph takes uint8 queries, a cosine graph float32 ones
    g.dtype = binding.U8
    with pytest.raises(TypeError):
        binding.query(g, ok_q, 10, 10, 0.3)
