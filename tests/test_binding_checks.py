"""The binding is the only place that can see a tensor's element type and size (the C ABI takes
plain pointers), so it must refuse a tensor that is narrower than the storage format named by
``dtype`` before anything is launched.  No GPU is needed: the checks run before the C call."""
import pytest
import torch

from paper_2601_12698_amd import binding as B


class FakeDeviceTensor:
    """Looks like a contiguous device tensor; a call that reached the library would dereference 0."""

    def __init__(self, dtype, numel):
        self.dtype, self._n = dtype, numel
        self.is_cuda = True
        self.device = None

    def numel(self):
        return self._n

    def element_size(self):
        return torch.empty(0, dtype=self.dtype).element_size()

    def is_contiguous(self):
        return True

    def data_ptr(self):
        raise AssertionError("the binding went on to marshal a tensor it should have refused")


M, N = 4, 256


@pytest.mark.parametrize("dtype,xt,rt,wt", [
    ("fp32", torch.bfloat16, torch.float32, torch.float32),       # x half as wide as the kernel would read
    ("fp32", torch.float32, torch.float16, torch.float32),
    ("fp16_res32", torch.float16, torch.float16, torch.float16),  # residual stream must be fp32
    ("fp16_res32", torch.float16, torch.float32, torch.float32),  # weight follows x
    ("bf16", torch.float16, torch.bfloat16, torch.bfloat16),      # same width, other format: wrong values, not refused by size
    ("fp16", torch.float16, torch.float16, torch.float32),
])
def test_addrms_run_refuses_mismatched_element_types(dtype, xt, rt, wt):
    x, r, w = FakeDeviceTensor(xt, M * N), FakeDeviceTensor(rt, M * N), FakeDeviceTensor(wt, N)
    with pytest.raises(ValueError, match="dtype asks for"):
        B.addrms_run(x, r, w, 1e-6, M, N, dtype)


def test_addrms_run_refuses_wrong_sizes_and_host_tensors():
    ok = lambda n: FakeDeviceTensor(torch.bfloat16, n)
    with pytest.raises(ValueError, match="elements, expected"):
        B.addrms_run(ok(M * N - 1), ok(M * N), ok(N), 1e-6, M, N, "bf16")
    with pytest.raises(ValueError, match="elements, expected"):
        B.addrms_run(ok(M * N), ok(M * N), ok(N + 1), 1e-6, M, N, "bf16")
    host = torch.zeros(M * N, dtype=torch.bfloat16)
    with pytest.raises(ValueError, match="device tensor"):
        B.addrms_run(host, host.clone(), torch.zeros(N, dtype=torch.bfloat16), 1e-6, M, N, "bf16")
    with pytest.raises(ValueError, match="unknown dtype"):
        B.addrms_run(ok(M * N), ok(M * N), ok(N), 1e-6, M, N, 17)


def test_silumul_and_mergestates_refuse_mismatched_element_types():
    with pytest.raises(ValueError, match="dtype asks for"):
        B.silumul_run(FakeDeviceTensor(torch.bfloat16, 2 * M * N), FakeDeviceTensor(torch.bfloat16, M * N), M, N, "fp32")
    with pytest.raises(ValueError, match="dtype asks for"):
        B.silumul_run(FakeDeviceTensor(torch.float16, 2 * M * N), FakeDeviceTensor(torch.bfloat16, M * N), M, N, "fp16")
    v = lambda: FakeDeviceTensor(torch.bfloat16, M * N)
    s32 = lambda: FakeDeviceTensor(torch.float32, M)
    with pytest.raises(ValueError, match="dtype asks for"):            # scores must be fp32
        B.mergestates_run(v(), FakeDeviceTensor(torch.bfloat16, M), v(), s32(), v(), s32(), M, N, "bf16")
    with pytest.raises(ValueError, match="dtype asks for"):
        B.mergestates_run(v(), s32(), FakeDeviceTensor(torch.float16, M * N), s32(), v(), s32(), M, N, "bf16")


def test_probes_refuse_mismatched_element_types():
    with pytest.raises(ValueError, match="dtype asks for"):
        B.addrms_stream_probe(FakeDeviceTensor(torch.float16, M * N), FakeDeviceTensor(torch.float16, M * N), M, N, "fp16_res32")
    y = lambda t: FakeDeviceTensor(t, M * N)
    counts = FakeDeviceTensor(torch.int32, 4)
    with pytest.raises(ValueError, match="dtype asks for"):
        B.addrms_gate_probe(y(torch.bfloat16), y(torch.bfloat16), y(torch.bfloat16), y(torch.bfloat16), "fp32", 1, counts)
    with pytest.raises(ValueError, match="elements, expected"):
        B.addrms_gate_probe(y(torch.float32), FakeDeviceTensor(torch.float32, 3), y(torch.float32), y(torch.float32), "fp32", 1, counts)
