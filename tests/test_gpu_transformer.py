"""Parity of the transformer-stage kernels (layer normalisation, causal attention, GELU, residual
connections, token + position embedding, per-position softmax cross-entropy) with the CPU oracle,
through the C ABI, with the same stage harness as tests/test_gpu_stage.py: forward of N micro-batches,
weights changed, one backward pass, update.  Shapes span the MFMA attention path (64 features per
head, several key blocks, a ragged last block) and the generic one (other head sizes, fp32).
"""
import numpy as np
import pytest

from tests.test_gpu_stage import run_stage_case
from workloads.configs import attention, embedding, layernorm, linear, softmax_ce, transformer_block

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d,rows,micro,N", [(64, 8, 3, 2), (768, 16, 4, 2), (100, 5, 7, 3)])
def test_layernorm_stage(dtype, d, rows, micro, N):
    run_stage_case([layernorm(d, rows), linear(d, 32, False, rows=rows)], dtype, micro, N, seed=d + rows)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("s,d,heads,micro,N", [
    (16, 32, 2, 2, 2),      # generic path: 16 features per head
    (40, 128, 2, 2, 2),     # 64 features per head, one ragged key block
    (200, 64, 1, 1, 2),     # several key blocks and a ragged tail
    (128, 192, 3, 2, 2),    # whole blocks, three heads
    (200, 256, 4, 12, 2),   # backward pass with four-wave workgroups
    (300, 768, 12, 12, 2),  # forward pass through the tiled kernel, backward pass with eight-wave workgroups, ragged
])
def test_attention_stage(dtype, s, d, heads, micro, N):
    # a linear layer in front so that the attention input gradient is used (and checked through dW as well)
    run_stage_case([linear(d, 3 * d, False, rows=s), attention(s, d, heads)], dtype, micro, N, seed=s + d)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_gelu_linear_pair(dtype):
    run_stage_case([linear(48, 96, False, act="gelu", rows=6), linear(96, 40, False, rows=6)], dtype, 5, 2, seed=21)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("s,d,heads,ffn", [(32, 64, 2, 128), (72, 128, 2, 256)])
def test_transformer_block_stage(dtype, s, d, heads, ffn):
    run_stage_case(transformer_block(s, d, heads, ffn), dtype, 2, 2, seed=s)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_embedding_block_stage(dtype):
    s, d = 24, 64
    run_stage_case([embedding(50, s, d)] + transformer_block(s, d, 1, 128), dtype, 3, 2, seed=31)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("vocab,s,micro,N", [(3, 64, 4, 2),      # every token some 170 times: more rows than the in-wave list holds
                                             (40, 48, 8, 2),     # a dozen rows per token
                                             (5000, 16, 4, 2)])  # most tokens absent, a few twice
def test_embedding_gradient_with_repeated_tokens(dtype, vocab, s, micro, N):
    # the token-table gradient adds the rows of a token in row order (no atomic adds): compared with the oracle, and
    # bit-identical between two passes over the same mini-batch
    import torch
    from paper_2410_14312_amd import Stage
    from tests.test_gpu_stage import _params
    d = 64
    specs = [embedding(vocab, s, d), linear(d, 32, False, rows=s)]
    run_stage_case(specs, dtype, micro, N, seed=vocab + s)
    rng = np.random.default_rng(7)
    st = Stage(specs, dtype, micro, N, N, 0.05, 0.9, device="cuda:0")
    st.set_params(_params(specs, rng))
    tok = torch.from_numpy(rng.integers(0, vocab, (micro * N, s)).astype(np.int32)).to(st.device)
    dy = torch.randn(micro * N, s * 32, dtype=torch.float32, device=st.device).to(st.act_dtype)
    seen = []
    for _ in range(2):
        for j in range(N):
            st.forward_micro(j, tok[j * micro:(j + 1) * micro])
        st.backward(list(range(N)), dy=dy)
        torch.cuda.synchronize()
        seen.append(st.get_grads()[0]["w"].copy())
    assert np.array_equal(seen[0], seen[1])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("borrow", [False, True])
def test_block_head_and_sequence_loss(dtype, borrow):
    s, d, vocab = 20, 64, 90
    specs = transformer_block(s, d, 2, 128) + [layernorm(d, s), linear(d, vocab, False, rows=s), softmax_ce(vocab, rows=s)]
    run_stage_case(specs, dtype, 2, 3, seed=41, borrow=borrow)


@pytest.mark.parametrize("name,stage", [("tiny_transformer_f32", 0), ("tiny_transformer_f32", 1),
                                        ("tiny_transformer_bf16", 0), ("tiny_transformer_bf16", 1)])
def test_tiny_transformer_config_stage(name, stage):
    from workloads import get_config
    cfg = get_config(name)
    run_stage_case(cfg.stages[stage], cfg.dtype, cfg.micro, cfg.N, seed=200 + stage, borrow=stage > 0)
