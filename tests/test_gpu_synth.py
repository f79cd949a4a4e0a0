"""The device twin of the counter-based input generator produces the CPU generator's bits."""
import numpy as np
import pytest

from paper_2410_10819_amd import binding as duo
from paper_2410_10819_amd import synth
from helpers import from_dev_bits

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("pos_start,n_pos,heads,d", [(0, 257, 8, 64), (123456, 100, 32, 128), (3299990, 10, 8, 128)])
def test_device_fill_matches_cpu(pos_start, n_pos, heads, d):
    import torch
    table = torch.from_numpy(synth.normal_table_bf16().view(np.int16)).cuda()
    for tensor_id, b in ((synth.TENSOR_K, 0), (synth.TENSOR_V, 3)):
        t = torch.zeros((n_pos, heads, d), dtype=torch.bfloat16, device="cuda")
        duo.duo_synth_fill_bf16(t, table, synth.stream_key(7, 5, tensor_id, b), pos_start, n_pos, heads, d)
        torch.cuda.synchronize()
        want = synth.counter_bf16(7, 5, tensor_id, b, pos_start, n_pos, heads, d)
        assert np.array_equal(from_dev_bits(t), want)
