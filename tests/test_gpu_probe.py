"""The streaming-read measurement aid (cafeq_stream_read_probe) reads its whole buffer: a lane writes the sink
only when the XOR of the words it read equals one constant, so in a buffer of zeros that constant planted in any one
word must set the sink (the vector holding it was read) and a buffer of zeros must not -- for lengths that end
inside a step of the kernel, inside a workgroup's share and below one step; the planted words include the first and
last vectors and both sides of the last, partial step."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2511_19705_amd import cafeq

pytestmark = pytest.mark.gpu
MAGIC = 0x5EEDF00D


@pytest.mark.parametrize("nvec", [1, 255, 1024, 1025, 4096 + 300, 8192 * 1024 + 777, 3 * 8192 * 1024 + 5])
def test_probe_reads_every_sampled_vector(nvec):
    rng = np.random.default_rng(nvec)
    dev = torch.device("cuda:0")
    buf = torch.zeros(4 * nvec, dtype=torch.int32, device=dev)
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    cafeq.stream_read_probe(buf, sink)
    torch.cuda.synchronize()
    assert int(sink.item()) == 0              # nothing read XORs to the constant
    tail0 = (nvec // 1024) * 1024             # first vector of the last, partial step
    vecs = {0, nvec - 1, nvec // 2, tail0 if tail0 < nvec else 0, max(tail0 - 1, 0), min(tail0 + 256, nvec - 1)}
    vecs |= {int(v) for v in rng.integers(0, nvec, size=6)}
    magic = MAGIC                             # (fits int32)
    for v in sorted(vecs):
        word = 4 * v + int(rng.integers(0, 4))
        buf[word] = magic
        sink.zero_()
        cafeq.stream_read_probe(buf, sink)
        torch.cuda.synchronize()
        assert int(sink.item()) & 0xFFFFFFFF == MAGIC, (nvec, v)
        buf[word] = 0


def test_probe_argument_errors():
    dev = torch.device("cuda:0")
    buf = torch.zeros(64, dtype=torch.int32, device=dev)
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    p = ctypes.c_void_p(buf.data_ptr())
    s = ctypes.c_void_p(sink.data_ptr())
    assert cafeq.lib.cafeq_stream_read_probe(None, ctypes.c_size_t(256), s, st) < 0
    assert cafeq.lib.cafeq_stream_read_probe(p, ctypes.c_size_t(256), None, st) < 0
    assert cafeq.lib.cafeq_stream_read_probe(p, ctypes.c_size_t(250), s, st) < 0
    assert cafeq.lib.cafeq_stream_read_probe(p, ctypes.c_size_t(0), s, st) < 0
    assert cafeq.lib.cafeq_stream_read_probe(ctypes.c_void_p(buf.data_ptr() + 4), ctypes.c_size_t(64), s, st) < 0
