"""duo_kv_append / duo_cache_export against the oracle's cache model: bit-exact."""
import numpy as np
import pytest

import oracle
from paper_2410_10819_amd import binding as duo
from paper_2410_10819_amd import synth
from helpers import to_dev, from_dev_bits

pytestmark = pytest.mark.gpu


def _export(handle, layer, b, h, d, fp8, capacity):
    """fp8: the cache's kv_dtype (0 bf16, 1 fp8: d code bytes + a scale, 2 int4: d/2 bytes + (scale, lo),
    3 int8: d bytes + (scale, lo))."""
    import torch
    if fp8:
        width = d // 2 if fp8 == 2 else d
        ko = torch.zeros((capacity, width), dtype=torch.uint8, device="cuda")
        vo = torch.zeros((capacity, width), dtype=torch.uint8, device="cuda")
        ks = torch.zeros((capacity, 2) if fp8 >= 2 else capacity, dtype=torch.float32, device="cuda")
        vs = torch.zeros((capacity, 2) if fp8 >= 2 else capacity, dtype=torch.float32, device="cuda")
    else:
        ko = torch.zeros((capacity, d), dtype=torch.bfloat16, device="cuda")
        vo = torch.zeros((capacity, d), dtype=torch.bfloat16, device="cuda")
        ks = vs = None
    po = torch.full((capacity,), -1, dtype=torch.int64, device="cuda")
    n = duo.duo_cache_export(handle, layer, b, h, ko, vo, po, capacity, kscale_out=ks, vscale_out=vs)
    torch.cuda.synchronize()
    pos = po[:n].cpu().numpy()
    if fp8:
        return pos, ko[:n].cpu().numpy(), vo[:n].cpu().numpy(), ks[:n].cpu().numpy(), vs[:n].cpu().numpy()
    return pos, from_dev_bits(ko[:n]), from_dev_bits(vo[:n]), None, None


@pytest.mark.parametrize("d,hkv,sink,recent,appends,fp8", [
    (64, 4, 1, 2, [4, 4, 4, 4], False),           # the figure's parameters
    (64, 4, 16, 64, [5, 1, 1, 90, 300, 1, 7], False),
    (128, 8, 64, 256, [1000, 1, 1, 1, 37], False),
    (128, 2, 0, 3, [2, 9, 1], False),
    (128, 8, 4, 8, [3, 40, 1, 1, 13], 1),
    (64, 4, 16, 64, [200, 1, 77], 1),
    (128, 8, 4, 8, [3, 40, 1, 1, 13], 2),
    (64, 4, 16, 64, [200, 1, 77], 2),
    (128, 8, 4, 8, [3, 40, 1, 1, 13], 3),
    (64, 4, 16, 64, [200, 1, 77], 3),
])
def test_append_then_export_matches_cache_model(d, hkv, sink, recent, appends, fp8):
    import torch
    batch, layers = 2, 2
    total = sum(appends)
    mask = synth.retrieval_mask(3, layers, hkv, 0.5)
    handle = duo.duo_cache_create(layers, batch, hkv, hkv, d, sink, recent, total + 5, mask, int(fp8))
    try:
        for layer in range(layers):
            k = synth.counter_bf16_batch(11, layer, synth.TENSOR_K, batch, 0, total, hkv, d)
            v = synth.counter_bf16_batch(11, layer, synth.TENSOR_V, batch, 0, total, hkv, d)
            if fp8:                      # exercise all-zero rows and exact powers of two
                k[0, 1, 0, :] = 0
                v[1, 2, 1, :] = 0
                k[0, 3, :, :] = synth.f32_to_bf16_bits(np.float32(0.5))
            models = [[oracle.CacheModel(sink, recent, bool(mask[layer, h])) for h in range(hkv)]
                      for _ in range(batch)]
            pos = 0
            for n in appends:
                duo.duo_kv_append(handle, layer, to_dev(k[:, pos:pos + n]), to_dev(v[:, pos:pos + n]), n)
                for b in range(batch):
                    for h in range(hkv):
                        for t in range(pos, pos + n):
                            models[b][h].append(k[b, t, h], v[b, t, h])
                pos += n
                assert duo.duo_cache_len(handle, layer) == pos
                for b in range(batch):
                    for h in range(hkv):
                        want_pos, want_k, want_v = models[b][h].contents()
                        assert want_pos == oracle.retained_positions(pos, sink, recent, bool(mask[layer, h]))
                        got_pos, gk, gv, gks, gvs = _export(handle, layer, b, h, d, fp8, total + 5)
                        assert got_pos.tolist() == want_pos
                        if not fp8:
                            assert np.array_equal(gk, want_k) and np.array_equal(gv, want_v)
                        elif fp8 >= 2:
                            quant = oracle.quantize_rows_int4 if fp8 == 2 else oracle.quantize_rows_int8
                            pack = oracle.pack_int4 if fp8 == 2 else (lambda c: c)
                            ck, sk, lk = quant(synth.bf16_bits_to_f32(want_k))
                            cv, sv, lv = quant(synth.bf16_bits_to_f32(want_v))
                            assert np.array_equal(gk, pack(ck)) and np.array_equal(gv, pack(cv))
                            for got_par, want_par in ((gks[:, 0], sk), (gks[:, 1], lk), (gvs[:, 0], sv), (gvs[:, 1], lv)):
                                assert np.array_equal(np.ascontiguousarray(got_par).view(np.uint32),
                                                      np.ascontiguousarray(want_par).view(np.uint32))
                        else:
                            ck, sk = oracle.quantize_rows(synth.bf16_bits_to_f32(want_k))
                            cv, sv = oracle.quantize_rows(synth.bf16_bits_to_f32(want_v))
                            assert np.array_equal(gk, ck) and np.array_equal(gv, cv)
                            assert np.array_equal(gks.view(np.uint32), sk.view(np.uint32))
                            assert np.array_equal(gvs.view(np.uint32), sv.view(np.uint32))
    finally:
        duo.duo_cache_destroy(handle)


def test_streaming_memory_is_constant_and_reset_works():
    hkv, d = 4, 64
    mask = np.array([[0, 0, 0, 0]], dtype=np.uint8)
    small = duo.duo_cache_create(1, 1, hkv, hkv, d, 16, 64, 1000, mask)
    large = duo.duo_cache_create(1, 1, hkv, hkv, d, 16, 64, 1000000, mask)
    try:
        assert duo.duo_cache_bytes(small) == duo.duo_cache_bytes(large) == 2 * hkv * 80 * d * 2
        k = synth.counter_bf16_batch(1, 0, synth.TENSOR_K, 1, 0, 10, hkv, d)
        duo.duo_kv_append(small, 0, to_dev(k), to_dev(k), 10)
        assert duo.duo_cache_len(small, 0) == 10
        duo.duo_cache_reset(small)
        assert duo.duo_cache_len(small, 0) == 0
    finally:
        duo.duo_cache_destroy(small)
        duo.duo_cache_destroy(large)


def test_runtime_errors_leave_the_handle_unchanged():
    import torch
    hkv, d = 2, 64
    mask = np.array([[1, 0]], dtype=np.uint8)
    h = duo.duo_cache_create(1, 1, 4, hkv, d, 4, 8, 16, mask)
    try:
        k = to_dev(synth.counter_bf16_batch(1, 0, synth.TENSOR_K, 1, 0, 17, hkv, d))
        q = to_dev(synth.counter_bf16_batch(1, 0, synth.TENSOR_Q, 1, 0, 1, 4, d))
        o = torch.empty((1, 1, 4, d), dtype=torch.bfloat16, device="cuda")
        with pytest.raises(duo.DuoError) as e:
            duo.duo_kv_append(h, 0, k, k, 17)
        assert e.value.status == duo.DUO_ERANGE
        with pytest.raises(duo.DuoError) as e:
            duo.duo_kv_append(h, 1, k, k, 1)
        assert e.value.status == duo.DUO_ERANGE
        with pytest.raises(duo.DuoError) as e:
            duo.duo_kv_append(h, 0, k, k, 0)
        assert e.value.status == duo.DUO_EINVAL
        with pytest.raises(duo.DuoError) as e:           # geometry disagrees with the cache
            duo.duo_kv_append(h, 0, k, k, 1, params=(None, 4, 9))
        assert e.value.status == duo.DUO_ESTATE
        with pytest.raises(duo.DuoError) as e:           # head classes disagree
            duo.duo_kv_append(h, 0, k, k, 1, params=(np.array([0, 0], np.uint8), 4, 8))
        assert e.value.status == duo.DUO_ESTATE
        with pytest.raises(duo.DuoError) as e:           # decode on an empty cache
            duo.duo_attn_decode(h, 0, q, o)
        assert e.value.status == duo.DUO_ESTATE
        assert duo.duo_cache_len(h, 0) == 0
        duo.duo_kv_append(h, 0, k[:, :16].contiguous(), k[:, :16].contiguous(), 16,
                          params=(np.array([1, 0], np.uint8), 4, 8))
        assert duo.duo_cache_len(h, 0) == 16
        with pytest.raises(duo.DuoError) as e:
            duo.duo_kv_append(h, 0, k, k, 1)
        assert e.value.status == duo.DUO_ERANGE
    finally:
        duo.duo_cache_destroy(h)
