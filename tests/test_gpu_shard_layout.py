"""The shard layout of the ring store (rtp_pack_shards / rtp_unpack_shards) against slots built from the oracle's
own splitting: bytes must be identical (integer / byte work: bit-exact), padding zero, the round trip exact."""
import ctypes as C

import numpy as np
import pytest
import torch

import rtp_workloads as wl
from paper_2311_01635_amd import binding as B
from paper_2311_01635_amd.layers import RtpLinear, RtpMlp
from slot_reference import matrix_parts, slots, vector_parts

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
_TD = {B.RTP_F32: torch.float32, B.RTP_BF16: torch.bfloat16, B.RTP_F16: torch.float16}


def _bits(t):
    """The raw storage of a tensor as a flat numpy array of unsigned integers of the element's size."""
    t = t.contiguous()
    return t.view(torch.int16 if t.element_size() == 2 else torch.int32).cpu().numpy().reshape(t.shape)


def _draw(shape, dtype, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(shape, dtype=np.float32)
    return torch.from_numpy(x).to(DEV, _TD[dtype])


@pytest.mark.parametrize("dtype", [B.RTP_BF16, B.RTP_F16, B.RTP_F32])
@pytest.mark.parametrize("split", [B.RTP_SPLIT_OUT, B.RTP_SPLIT_IN])
@pytest.mark.parametrize("O,I,n", [(96, 40, 4), (40, 96, 8), (1000, 72, 8), (72, 1000, 8), (333, 517, 7), (64, 64, 1)])
def test_pack_matches_the_oracles_split_and_unpack_inverts_it(O, I, n, split, dtype):
    part = O if split == B.RTP_SPLIT_OUT else I
    w = B.lib.rtp_shard_width(part, n, dtype)
    if w <= 0:
        pytest.skip("this dimension cannot be split into n non-empty aligned shards")
    es = 4 if dtype == B.RTP_F32 else 2
    other = I if split == B.RTP_SPLIT_OUT else O
    lead, tail = 16 // es * 3, 16 // es * 2                         # the part sits inside a larger slot
    slot_elems = lead + w * other + tail
    W = _draw((O, I), dtype, seed=O + 3 * I + n)
    home = torch.full((n, slot_elems), 7.0, dtype=_TD[dtype], device=DEV)   # whatever is around the part stays
    print(f"pack O={O} I={I} n={n} split={split} dtype={dtype} width={w}", flush=True)
    B.rtp_pack_shards(home, slot_elems * es, lead * es, n, split, W, O, I, w, dtype)
    torch.cuda.synchronize()
    want = slots(n, slot_elems, [(lead, matrix_parts(_bits(W), n, split == B.RTP_SPLIT_OUT, w))])
    got = _bits(home)
    seven = _bits(torch.full((1,), 7.0, dtype=_TD[dtype]))[0]
    want[:, :lead] = seven
    want[:, lead + w * other:] = seven
    assert np.array_equal(got, want)
    back = torch.full((O, I), float("nan"), dtype=_TD[dtype], device=DEV)
    B.rtp_unpack_shards(back, home, slot_elems * es, lead * es, n, split, O, I, w, dtype)
    torch.cuda.synchronize()
    assert np.array_equal(_bits(back), _bits(W))


def test_linear_layer_store_is_the_oracles_partition():
    """RtpLinear builds its stores through the library: weights [W_k | bias entries], gradients the same in fp32,
    for both partitions, with a partition that needs padding."""
    O, I, n, T = 232, 184, 6, 32      # 6 divides neither: both partitions are padded (widths 40 and 32)
    W, b = _draw((O, I), B.RTP_BF16, 1), _draw((O,), B.RTP_BF16, 2)
    G0 = _draw((O, I), B.RTP_F32, 3)
    for split in (B.RTP_SPLIT_OUT, B.RTP_SPLIT_IN):
        layer = RtpLinear(W, T, n, 2, split, B.RTP_DOUBLE_BUFFER, B.RTP_BF16, G0=G0, bias=b)
        w = layer.o
        n_mat = w * (I if split == B.RTP_SPLIT_OUT else O)
        pw = w if split == B.RTP_SPLIT_OUT else B.lib.rtp_bias_piece_width(O, n, B.RTP_BF16)
        want_w = slots(n, layer.home_w.shape[1] // 2, [(0, matrix_parts(_bits(W), n, split == B.RTP_SPLIT_OUT, w)),
                                                      (n_mat, vector_parts(_bits(b), n, pw))])
        want_g = slots(n, layer.home_g.shape[1] // 4, [(0, matrix_parts(_bits(G0), n, split == B.RTP_SPLIT_OUT, w)),
                                                      (n_mat, vector_parts(np.zeros(O, dtype=np.int32), n, pw))])
        assert np.array_equal(layer.home_w.view(torch.int16).cpu().numpy(), want_w), split
        assert np.array_equal(layer.home_g.view(torch.int32).cpu().numpy(), want_g), split
        layer.close()


@pytest.mark.parametrize("gated", [False, True])
def test_mlp_unit_slot_is_gate_up_down_back_to_back(gated):
    """Slot k of the MLP unit = [W1_k | W2_k] or [gate_k ; up_k | down_k], every part the oracle's shard."""
    T, I, O, O2, n = 64, 72, 8 * 24, 40, 8
    names = ("Wg", "Wu", "Wd") if gated else ("W1", "W2")
    shapes = [(O, I)] * (2 if gated else 1) + [(O2, O)]
    Ws = [_draw(sh, B.RTP_BF16, 10 + i) for i, sh in enumerate(shapes)]
    G0 = [_draw(sh, B.RTP_F32, 20 + i) for i, sh in enumerate(shapes)]
    act = B.RTP_ACT_SWIGLU if gated else B.RTP_ACT_GELU_ERF
    mlp = RtpMlp(Ws, T, n, 1, act, B.RTP_INPLACE_STAGED, B.RTP_BF16, G0=G0)
    o, p = O // n, len(shapes) - 1
    for home, mats, view, es in ((mlp.home_w, Ws, torch.int16, 2), (mlp.home_g, G0, torch.int32, 4)):
        placed = [(j * o * I, matrix_parts(_bits(mats[j]), n, True, o)) for j in range(p)]
        placed.append((p * o * I, matrix_parts(_bits(mats[-1]), n, False, o)))
        want = slots(n, home.shape[1] // es, placed)
        assert np.array_equal(home.view(view).cpu().numpy(), want), names
    Wb, Gb = mlp.gathered()
    for a, b_ in zip(Wb, Ws):
        assert torch.equal(a, b_)
    for a, b_ in zip(Gb, G0):
        assert torch.equal(a, b_)
    mlp.close()
