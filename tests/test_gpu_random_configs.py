"""Parity on seeded random configurations: shapes, window geometry, chunkings, head classes, cache
types, decode kernels and split counts drawn at random (a fixed list, the same in every run), every
output element against the float64 oracle.  The hand-picked cases of the other files aim at known
borders; these look for the ones nobody thought of."""
import numpy as np
import pytest

from paper_2410_10819_amd import binding as duo
from paper_2410_10819_amd import synth
from helpers import ATOL_LSE, assert_close, make_qkv, oracle_rows, run_scenario
from test_gpu_attention import _check_all, _decode_vs_oracle

pytestmark = pytest.mark.gpu


def _draw_shape(rng):
    hkv = int(rng.choice([1, 2, 3, 4, 8]))
    group = int(rng.choice([1, 1, 2, 4, 8]))
    d = int(rng.choice([64, 128]))
    sink = int(rng.integers(0, 41))
    recent = int(rng.choice([1, 2, 7, 31, 32, 33, 64, 100]))
    mask = rng.integers(0, 2, size=hkv).astype(np.uint8)
    return hkv, group, d, sink, recent, mask


def _draw_wide_shape(rng):
    """Like _draw_shape with sink counts and windows of several tiles (and windows longer than the fill)."""
    hkv, group, d, _, _, mask = _draw_shape(rng)
    sink = int(rng.choice([0, 63, 64, 65, 128, 200, 300]))
    recent = int(rng.choice([127, 128, 129, 256, 300, 511, 600]))
    return hkv, group, d, sink, recent, mask


def _decode_cases():
    rng = np.random.default_rng(20241010)
    cases = []
    for i in range(34):
        hkv, group, d, sink, recent, mask = _draw_shape(rng) if i < 24 else _draw_wide_shape(rng)
        kv_dtype = int(rng.choice([0, 0, 0, 1, 2, 3]))
        batch = int(rng.integers(1, 4))
        n_fill = int(rng.choice([0, 1, 31, 32, 33, 200, 777, 1500, 2600]))
        # the vector-unit kernel serves one query head per KV head on bf16 rows; anything else runs on the
        # matrix-core kernel anyway, and half of the eligible cases are forced onto it as well
        kernel = int(rng.integers(0, 2)) if (group == 1 and kv_dtype == 0) else 0
        splits = int(rng.choice([0, 0, 1, 3, 7]))
        cases.append(pytest.param(hkv * group, hkv, d, sink, recent, batch, n_fill, kv_dtype, mask, kernel, splits, i,
                                  id="%d-h%dx%d-d%d-s%d-r%d-b%d-n%d-kv%d-k%d-sp%d" % (
                                      i, hkv, group, d, sink, recent, batch, n_fill, kv_dtype, kernel, splits)))
    return cases


@pytest.mark.parametrize("hq,hkv,d,sink,recent,batch,n_fill,kv_dtype,mask,kernel,splits,seed", _decode_cases())
def test_random_decode_configurations(hq, hkv, d, sink, recent, batch, n_fill, kv_dtype, mask, kernel, splits, seed):
    _decode_vs_oracle(hq, hkv, d, sink, recent, batch, n_fill, 3, kv_dtype, mask, kernel=kernel, splits=splits,
                      seed=1000 + seed)


def _prefill_cases():
    rng = np.random.default_rng(20241011)
    cases = []
    for i in range(22):
        hkv, group, d, sink, recent, mask = _draw_shape(rng) if i < 14 else _draw_wide_shape(rng)
        batch = int(rng.integers(1, 3))
        total = int(rng.integers(40, 1300))
        n_chunks = int(rng.integers(1, 6))
        cuts = np.sort(rng.choice(np.arange(1, total), size=min(n_chunks - 1, total - 1), replace=False))
        chunks = np.diff(np.concatenate([[0], cuts, [total]])).astype(int).tolist()
        deployed = bool(rng.integers(0, 2))
        cases.append(pytest.param(hkv * group, hkv, d, sink, recent, batch, chunks, mask, deployed, i,
                                  id="%d-h%dx%d-d%d-s%d-r%d-b%d-%s-%s" % (
                                      i, hkv, group, d, sink, recent, batch, "+".join(map(str, chunks)),
                                      "deployed" if deployed else "lambda")))
    return cases


@pytest.mark.parametrize("hq,hkv,d,sink,recent,batch,chunks,mask,deployed,seed", _prefill_cases())
def test_random_prefill_configurations(hq, hkv, d, sink, recent, batch, chunks, mask, deployed, seed):
    total, n_decode = sum(chunks), 2
    cfg = dict(batch=batch, hq=hq, hkv=hkv, d=d, sink=sink, recent=recent, mask=mask, max_seq=total + n_decode)
    q, k, v = make_qkv(2000 + seed, batch, total + n_decode, hq, hkv, d)
    out, lse, handle = run_scenario(duo, cfg, q, k, v, chunks, n_decode, deployed=deployed,
                                    fused_decode="step" if seed % 2 else False)
    duo.duo_cache_destroy(handle)
    if not deployed:
        _check_all(cfg, q, k, v, out, lse)
        return
    starts = np.concatenate([np.full(n, p) for p, n in zip(np.cumsum([0] + chunks[:-1]), chunks)])
    for b in range(batch):
        want_o, want_lse = oracle_rows(cfg, q, k, v, np.arange(total), b, chunk_starts=starts)
        assert_close(synth.bf16_bits_to_f64(out[b][:total]), want_o, "deployed prefill, batch %d" % b)
        assert np.abs(lse[b][:, :total] - want_lse).max() <= ATOL_LSE
        want_d, _ = oracle_rows(cfg, q, k, v, np.arange(total, total + n_decode), b)
        assert_close(synth.bf16_bits_to_f64(out[b][total:]), want_d, "decode after deployed prefill")


def _gate_cases():
    rng = np.random.default_rng(20241012)
    cases = []
    for i in range(8):
        hkv, group, d, sink, recent, _ = _draw_shape(rng)
        t = int(rng.integers(20, 900))
        block = int(rng.choice([0, 0, 1, 5, 16, 64, 128]))
        batch = int(rng.integers(1, 3))
        alpha = rng.uniform(0, 1, hkv).astype(np.float32)
        alpha[int(rng.integers(0, hkv))] = float(rng.integers(0, 2))    # one gate at an end of the range
        cases.append(pytest.param(hkv * group, hkv, d, sink, recent, batch, t, alpha, block, i,
                                  id="%d-h%dx%d-d%d-s%d-r%d-b%d-t%d-blk%d" % (i, hkv, group, d, sink, recent, batch, t, block)))
    return cases


@pytest.mark.parametrize("hq,hkv,d,sink,recent,batch,t,alpha,block,seed", _gate_cases())
def test_random_gate_mixed_configurations(hq, hkv, d, sink, recent, batch, t, alpha, block, seed):
    from test_gpu_gate_mixed import _run
    _run(hq, hkv, d, sink, recent, batch, t, alpha, block, seed=3000 + seed)


def _cache_cases():
    rng = np.random.default_rng(20241013)
    cases = []
    for i in range(8):
        hkv, _, d, sink, recent, _ = _draw_shape(rng)
        kv_dtype = int(rng.integers(0, 4))
        appends = [int(x) for x in rng.choice([1, 1, 2, 5, 33, 64, 150, 400], size=int(rng.integers(2, 6)))]
        cases.append(pytest.param(d, hkv, sink, recent, appends, kv_dtype,
                                  id="%d-h%d-d%d-s%d-r%d-kv%d-%s" % (i, hkv, d, sink, recent, kv_dtype,
                                                                     "+".join(map(str, appends)))))
    return cases


@pytest.mark.parametrize("d,hkv,sink,recent,appends,kv_dtype", _cache_cases())
def test_random_append_sequences_leave_the_model_contents(d, hkv, sink, recent, appends, kv_dtype):
    from test_gpu_cache import test_append_then_export_matches_cache_model as check
    check(d, hkv, sink, recent, appends, kv_dtype)
