"""Host-side checks of the Python binding and the modules that need no GPU: the binding refuses
tensors whose dtype or size the C ABI would misread, before anything reaches the device, and
the LayerNorm module keeps its parameters in float32 whatever the model is cast to."""
import pytest
import torch

from paper_2210_10246_amd import binding as B
from paper_2210_10246_amd.modules import InplaceLayerNorm, TempoEncoderLayer


def test_layernorm_parameters_must_be_float32():
    x = torch.zeros(4, 64, dtype=torch.bfloat16)
    y = torch.empty_like(x)
    rstd = torch.empty(4, dtype=torch.float32)
    g16 = torch.ones(64, dtype=torch.bfloat16)
    g32 = torch.ones(64, dtype=torch.float32)
    with pytest.raises(ValueError, match="gamma"):
        B.tempo_layernorm_fwd(x, g16, g32, y, rstd)
    with pytest.raises(ValueError, match="beta"):
        B.tempo_layernorm_fwd(x, g32, g16, y, rstd)
    with pytest.raises(ValueError, match="rstd"):
        B.tempo_layernorm_fwd(x, g32, g32, y, rstd.double())
    with pytest.raises(ValueError, match="rstd"):
        B.tempo_layernorm_fwd(x, g32, g32, y, rstd[:3])
    with pytest.raises(ValueError, match="gamma"):
        B.tempo_layernorm_fwd(x, g32[:32], g32, y, rstd)
    ws = torch.empty(1 << 16, dtype=torch.uint8)
    with pytest.raises(ValueError, match="dgamma"):
        B.tempo_layernorm_bwd(x, y, g32, g32, rstd, y, g16, g32, ws)
    with pytest.raises(ValueError, match="dy"):
        B.tempo_layernorm_bwd(x.float(), y, g32, g32, rstd, y, g32, g32, ws)


def test_masks_key_len_and_activations_are_checked():
    x = torch.zeros(100, dtype=torch.float32)
    with pytest.raises(ValueError, match="mask"):
        B.tempo_gelu_fwd(x, x, torch.zeros(4, dtype=torch.int64))
    with pytest.raises(ValueError, match="mask"):
        B.tempo_gelu_fwd(x, x, torch.zeros(3, dtype=torch.int32))     # needs ceil(100/32) = 4 words
    with pytest.raises(ValueError, match="float32 or bfloat16"):
        B.tempo_gelu_fwd(x.half(), x.half(), torch.zeros(4, dtype=torch.int32))
    with pytest.raises(ValueError, match="dy"):
        B.tempo_silu_bwd(x.bfloat16(), x, torch.zeros(4, dtype=torch.int32), x)
    s = torch.zeros(2, 1, 4, 8, dtype=torch.float32)
    keep = torch.zeros(2, dtype=torch.int32)
    with pytest.raises(ValueError, match="key_len"):
        B.tempo_attn_softmax_dropout_fwd(s, torch.tensor([8, 8]), False, s, s, keep, 0.1, 1, 0)   # int64
    with pytest.raises(ValueError, match="key_len"):
        B.tempo_attn_softmax_dropout_fwd(s, torch.tensor([8], dtype=torch.int32), False, s, s, keep, 0.1, 1, 0)
    with pytest.raises(ValueError, match="keep_bits"):
        B.tempo_attn_softmax_dropout_bwd(s, s, keep[:1], s, None, 0.1)
    with pytest.raises(ValueError, match="dout"):
        B.tempo_attn_softmax_dropout_bwd_regen(s.bfloat16(), s, s, None, 0.1, 1, 0)


def test_layernorm_module_keeps_float32_parameters_under_casts():
    layer = TempoEncoderLayer(64, 4, 256)
    with torch.no_grad():
        layer.ln1.weight.add_(0.123456789)
    w0 = layer.ln1.weight.detach().clone()
    layer = layer.bfloat16()
    assert layer.fc1.weight.dtype == torch.bfloat16
    assert layer.ln1.weight.dtype == torch.float32 and layer.ln2.bias.dtype == torch.float32
    assert torch.equal(layer.ln1.weight, w0)              # values untouched, not rounded to bf16
    assert isinstance(layer.ln1.weight, torch.nn.Parameter)
    layer = layer.to(torch.float16)
    assert layer.ln1.weight.dtype == torch.float32
    ln = InplaceLayerNorm(8).double()
    assert ln.weight.dtype == torch.float32
