"""GPU parity of transformer-shaped stages against the fp64 oracle: layer normalisation, per-token dense
layers, causal multi-head attention and residual connections, driven like the other single-stage tests
(forward, backward with real staleness under the blend, update), in both precisions."""
import pytest

from synth_inputs import workloads as W
from stage_parity import run_stage as _run_stage

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_layernorm_and_per_token_dense(dtype):
    # 7 tokens x 24 features (no multiple of anything), LN -> dense+GELU -> LN -> dense
    specs = (W.LayerNorm(24, 7), W.Dense(24, 40, "gelu", tokens=7), W.LayerNorm(40, 7), W.Dense(40, 16, "none", tokens=7))
    print(dtype, _run_stage(specs, f"ln_{dtype}", dtype, mb=3, n=2))


def test_layernorm_wide_rows_bf16():
    # widths 512 and 1536: the register-resident bf16 normalisation kernels (rows of 1 and 3 groups per lane)
    specs = (W.LayerNorm(512, 5), W.Dense(512, 1536, "gelu", tokens=5), W.LayerNorm(1536, 5), W.Dense(1536, 64, "none", tokens=5))
    print(_run_stage(specs, "ln_wide", "bf16", mb=3, n=2))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_attention_alone(dtype):
    # qkv projection -> attention -> output projection; 21 tokens: ragged against the 16-row / 64-key tiles
    specs = (W.Dense(16, 48, "none", tokens=21), W.Attention(16, 2, 21), W.Dense(16, 16, "none", tokens=21))
    print(dtype, _run_stage(specs, f"attn_{dtype}", dtype, mb=2, n=2))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_residual_around_gelu_dense(dtype):
    # the residual add follows an activation and the begin follows one too
    specs = (W.Dense(16, 16, "gelu", tokens=4), W.Residual(16, 4, "begin"), W.Dense(16, 16, "gelu", tokens=4),
             W.Residual(16, 4, "add"), W.Dense(16, 8, "none", tokens=4))
    print(dtype, _run_stage(specs, f"res_{dtype}", dtype, mb=3, n=2))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_two_transformer_blocks(dtype):
    # two pre-norm decoder blocks, 80 tokens (two key tiles), 4 heads of 8, depth 3: staleness 0, 1, 2
    specs = W.transformer_block(32, 4, 64, 80) + W.transformer_block(32, 4, 64, 80)
    print(dtype, _run_stage(specs, f"tfm2_{dtype}", dtype, mb=2, n=2, depth=3, minibatches=4))


def test_transformer_block_first_stage_no_input_gradient():
    specs = W.transformer_block(32, 2, 64, 16)
    print(_run_stage(specs, "tfm_first", "f32", mb=2, n=2, needs_dx=False))


def test_transformer_block_wide_heads_bf16():
    # head width 128 (two output columns per lane in the attention kernels), 128-wide model, 64 tokens
    specs = W.transformer_block(128, 1, 256, 64)
    print(_run_stage(specs, "tfm_wide", "bf16", mb=2, n=2))


def test_attention_matrix_core_ragged_tiles_bf16():
    # 192 tokens (one and a half 128-row tiles), 3 heads of 64: the matrix-core attention with a ragged
    # last tile, causal tile skipping and both contraction shortcuts; projections around it
    specs = (W.Dense(64, 3 * 192, "none", tokens=192), W.Attention(192, 3, 192), W.Dense(192, 64, "none", tokens=192))
    print(_run_stage(specs, "attn_mfma", "bf16", mb=2, n=2))


def test_transformer_stage_reduced_bf16():
    # the decoder stage of the transformer workload at reduced size: 4 blocks (44 layers), d_model 256,
    # 4 heads of 64, FFN 1024, 128 tokens, micro-batch 2 x 2, depth 3 (staleness 0, 1, 2)
    w = W.transformer_stage(d=256, heads=4, ffn=1024, tokens=128, layers=4, mb=2, n=2)
    print(_run_stage(w.stages[1], "tfm_reduced", "bf16", mb=2, n=2, depth=3, minibatches=3))


@pytest.mark.parametrize("tokens,heads,dh", [(64, 2, 64), (192, 1, 128), (320, 2, 64), (512, 1, 128)])
def test_fused_attention_bf16(tokens, heads, dh):
    # the fused forward and backward kernels: one 64-row block (two of the waves at work), partly filled workgroups,
    # several workgroups per head with different numbers of blocks to walk (320 = 256 + 64 = 128 + 128 + 64), several
    # diagonal blocks; head widths 64 and 128.  The projections around it make the inputs and the upstream gradient
    # ordinary.
    d = heads * dh
    specs = (W.Dense(32, 3 * d, "none", tokens=tokens), W.Attention(d, heads, tokens), W.Dense(d, 32, "none", tokens=tokens))
    print(tokens, heads, dh, _run_stage(specs, f"attn_flash_{tokens}_{heads}_{dh}", "bf16", mb=2, n=2))
