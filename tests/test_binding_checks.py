"""The Python binding refuses buffers that are too small, of the wrong type or not on the
device before anything reaches the C ABI (which sees plain pointers and cannot check sizes).
No GPU needed: the refusals come before the first device call."""
import numpy as np
import pytest
import torch

from paper_2412_01195_amd import q8opt


def _bufs(n, B, short=None):
    nb = -(-n // B)
    sizes = dict(w=n, g=n, m_q=n, r_q=n, N_m=nb, N_r=nb)
    if short:
        sizes[short] -= 1
    f = lambda k, dt: torch.zeros(sizes[k], dtype=dt)
    return dict(w=f("w", torch.float32), g=f("g", torch.float32), m_q=f("m_q", torch.uint8), r_q=f("r_q", torch.uint8),
                N_m=f("N_m", torch.float32), N_r=f("N_r", torch.float32))


def _tab():
    return torch.zeros(q8opt.qtable_bytes(), dtype=torch.uint8)


@pytest.mark.parametrize("short", ["g", "m_q", "r_q", "N_m", "N_r"])
def test_adam_refuses_short_buffers(short):
    b = _bufs(5000, 2048, short)
    with pytest.raises(ValueError, match=short + " holds"):
        q8opt.adam8bit_step(b["w"], b["g"], b["m_q"], b["r_q"], b["N_m"], b["N_r"], _tab(), _tab(), 2048,
                            1e-3, 0.9, 0.999, 1e-8)


def test_full_size_host_tensors_are_refused_as_not_on_the_device():
    b = _bufs(5000, 2048)
    with pytest.raises(ValueError, match="CUDA"):
        q8opt.adam8bit_step(b["w"], b["g"], b["m_q"], b["r_q"], b["N_m"], b["N_r"], _tab(), _tab(), 2048,
                            1e-3, 0.9, 0.999, 1e-8)


def test_wrong_type_and_short_table():
    b = _bufs(4096, 2048)
    with pytest.raises(ValueError, match="dtype"):
        q8opt.sgd8bit_step(b["w"], b["g"].double(), b["m_q"], b["N_m"], _tab(), 2048, 0.1, 0.9)
    with pytest.raises(ValueError, match="qtable_signed holds"):
        q8opt.sgd8bit_step(b["w"], b["g"], b["m_q"], b["N_m"], _tab()[:-1], 2048, 0.1, 0.9)
    with pytest.raises(ValueError, match="N holds"):
        q8opt.quantize_blockwise(_tab(), b["w"], 2048, b["m_q"], b["N_m"][:1])
    with pytest.raises(ValueError, match="TD holds"):
        q8opt.dequantize_blockwise(_tab(), b["m_q"], b["N_m"], 2048, b["w"][:100])


def test_list_entries_are_checked_one_by_one():
    good, bad = _bufs(3000, 256), _bufs(3000, 256, "N_r")
    with pytest.raises(ValueError, match="tensor 1: N_r holds"):
        q8opt.Plan([good, bad], 256)
    small = dict(w=torch.zeros(100), g=torch.zeros(100), m_f32=torch.zeros(100), r_f32=torch.zeros(99))
    with pytest.raises(ValueError, match="tensor 0: r_f32 holds"):
        q8opt.multi_adam8bit_step_noalloc([small], 256, _tab(), _tab(), 1e-3, 0.9, 0.999, 1e-8)
