"""cake_quantize_kv against the oracle's quantiser on the compacted caches of a real pass: codes,
scales and zero points bit for bit (both sides decide the codes in float32), the packing of
codes into bytes, ragged batches, a last token group that is not full, untouched rows beyond a
sequence's own count, and the half-step reconstruction bound."""
import numpy as np
import pytest
import torch

from oracle import cake_oracle as co
from synth import CONFIGS, make_config_inputs

from gpu_util import load_cake, say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def cake():
    return load_cake()


def _unpack(codes_bytes: np.ndarray, bits: int) -> np.ndarray:
    """[rows, d*bits/8] uint8 -> [rows, d] codes: 8/bits consecutive channels per byte, lower channel in the lower bits."""
    per = 8 // bits
    parts = [(codes_bytes >> (i * bits)) & ((1 << bits) - 1) for i in range(per)]
    return np.stack(parts, axis=-1).reshape(codes_bytes.shape[0], -1)


def _check(cake, cfg, bits):
    inp = make_config_inputs(cfg, device=DEV)
    L = cfg.n_layers
    res = cake.EvictionPass([inp["q_win"][l] for l in range(L)], [inp["k"][l] for l in range(L)],
                            [inp["v"][l] for l in range(L)], cfg.total_budget).run()
    torch.cuda.synchronize()
    quant = cake.CacheQuantizer(res, cfg.window, bits)
    for t in quant.out.k_codes + quant.out.v_codes:
        t.fill_(0xA5)                                   # rows beyond a sequence's own count must keep this
    out = quant.run()
    torch.cuda.synchronize()
    worst = 0.0
    for l in range(L):
        for b in range(cfg.batch):
            n_k = int(res.keep[l, b])
            cap = int(res.keep[l].max())
            for g in range(cfg.n_kv_heads):
                k_rows = res.k_out[l][b, g, :n_k].float().cpu().numpy()
                v_rows = res.v_out[l][b, g, :n_k].float().cpu().numpy()
                if n_k:
                    (kc, ks, kz), (vc, vs, vz) = co.quantize_cache(k_rows, v_rows, bits)
                    np.testing.assert_array_equal(_unpack(out.k_codes[l][b, g, :n_k].cpu().numpy(), bits), kc)
                    np.testing.assert_array_equal(_unpack(out.v_codes[l][b, g, :n_k].cpu().numpy(), bits), vc)
                    ng = -(-n_k // 32)
                    np.testing.assert_array_equal(out.k_scale[l][b, g, :ng].cpu().numpy(), ks)
                    np.testing.assert_array_equal(out.k_zero[l][b, g, :ng].cpu().numpy(), kz)
                    np.testing.assert_array_equal(out.v_scale[l][b, g, :n_k].cpu().numpy(), vs)
                    np.testing.assert_array_equal(out.v_zero[l][b, g, :n_k].cpu().numpy(), vz)
                    back = co.dequantize_uniform(kc, ks, kz, 0)
                    half = np.repeat(ks, 32, axis=0)[:n_k] / 2
                    assert np.all(np.abs(back - k_rows) <= half * (1 + 1e-5) + 1e-6)
                    worst = max(worst, float(np.abs(back - k_rows).max()))
                if n_k < cap:                           # ragged batch: the rest of the capacity is untouched
                    assert (out.k_codes[l][b, g, n_k:cap] == 0xA5).all() and (out.v_codes[l][b, g, n_k:cap] == 0xA5).all()
    say(f"  {bits}-bit: largest key reconstruction error {worst:.4f}")


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_quantised_cache_equals_the_oracle_llama_shape(cake, bits):
    say(f"quantise bf16 d = 128, {bits} bits")
    _check(cake, CONFIGS[2].scaled(n_layers=3, seq_len=1500, total_budget=3 * 333), bits)


def test_quantised_cache_equals_the_oracle_ragged_batch_and_fp32(cake):
    say("quantise: batch of 3 with per-sequence counts (bf16), tiny fp32 d = 64")
    _check(cake, CONFIGS[5].scaled(n_layers=2, batch=3, seq_len=900, total_budget=2 * 170), 4)
    _check(cake, CONFIGS[1], 4)
    _check(cake, CONFIGS[1], 2)


def test_quantiser_rounding_boundaries(cake):
    # Every group holds 0 and 2^b - 1, so its scale is exactly 1 and the quotients are the values
    # themselves: exact ties k + 1/2 (round-half-even) and their nearest representable neighbours,
    # where a product with a rounded reciprocal could fall on the other side of the boundary.
    from types import SimpleNamespace
    say("quantise: values on and next to the rounding boundaries")
    rng = np.random.default_rng(7)
    for bits, dtype in ((4, torch.bfloat16), (8, torch.bfloat16), (2, torch.float32), (8, torch.float32)):
        levels, d, rows, window, H = 2 ** bits - 1, 128, 70, 32, 2
        top = min(levels, 127)                                        # k + 1/2 is a bf16 number up to 127.5
        def tile():
            x = torch.from_numpy(rng.integers(0, top, size=(H, rows, d)).astype(np.float32) + 0.5).to(dtype)
            step = torch.from_numpy(rng.choice([-1, 0, 0, 1], size=(H, rows, d)))      # units in the last place of dtype
            as_int = torch.int16 if dtype == torch.bfloat16 else torch.int32
            x = (x.view(as_int) + step.to(as_int)).view(dtype)                          # positive values: the neighbouring numbers
            return x.float().numpy()                                                    # what the device will hold
        k, v = tile(), tile()
        k[:, 0::32] = 0.0; k[:, 1::32] = levels                       # per channel, in every token group
        v[:, :, 0::32] = 0.0; v[:, :, 1::32] = levels                 # per token, in every channel group
        pad = np.zeros((H, window, d), np.float32)
        to_dev = lambda x: torch.from_numpy(np.concatenate([x, pad], axis=1)[None]).to(dtype).to(DEV)
        res = SimpleNamespace(keep=np.array([[rows]]), k_out=[to_dev(k)], v_out=[to_dev(v)])
        out = cake.CacheQuantizer(res, window, bits).run()
        torch.cuda.synchronize()
        ties = 0
        for g in range(H):
            (kc, ks, kz), (vc, vs, vz) = co.quantize_cache(k[g], v[g], bits)
            assert np.all(ks == 1.0) and np.all(vs == 1.0) and np.all(kz == 0.0) and np.all(vz == 0.0)
            np.testing.assert_array_equal(_unpack(out.k_codes[0][0, g, :rows].cpu().numpy(), bits), kc)
            np.testing.assert_array_equal(_unpack(out.v_codes[0][0, g, :rows].cpu().numpy(), bits), vc)
            np.testing.assert_array_equal(out.k_scale[0][0, g, :3].cpu().numpy(), ks)
            np.testing.assert_array_equal(out.v_zero[0][0, g, :rows].cpu().numpy(), vz)
            ties += int(np.sum(k[g] - np.floor(k[g]) == 0.5)) + int(np.sum(v[g] - np.floor(v[g]) == 0.5))
        assert ties > 1000
        say(f"  {bits}-bit {dtype}: {ties} exact ties among {2 * H * rows * d} values")


def test_quantiser_rejects_bad_arguments(cake):
    from paper_2503_12491_amd import binding as C
    cfg = CONFIGS[1]
    inp = make_config_inputs(cfg, device=DEV)
    L = cfg.n_layers
    res = cake.EvictionPass([inp["q_win"][l] for l in range(L)], [inp["k"][l] for l in range(L)],
                            [inp["v"][l] for l in range(L)], cfg.total_budget).run()
    torch.cuda.synchronize()
    q = cake.CacheQuantizer(res, cfg.window, 4)
    for bits in (0, 3, 16):
        with pytest.raises(C.CakeError):
            C.cake_quantize_kv(q.shape, bits, q.tbl[0], q.tbl[1], q.strides, q.keep_flat, *q.tbl[2:])
    with pytest.raises(C.CakeError):
        C.cake_quantize_kv(q.shape, 4, q.tbl[0], q.tbl[1], q.strides, [-1] * len(q.keep_flat), *q.tbl[2:])
    with pytest.raises(C.CakeError):
        C.cake_quantize_kv(q.shape, 4, None, q.tbl[1], q.strides, q.keep_flat, *q.tbl[2:])
    torch.cuda.synchronize()
