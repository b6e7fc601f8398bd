"""Host logic: which FFN kernel the library picks for the shapes the bench runs
(no GPU needed: moe_ffn_kernel_name only evaluates the selection rules)."""
import pytest

from workloads import get_config


@pytest.fixture(scope="module")
def B():
    import os
    for v in ("MOE_TUNE_BLOCK", "MOE_TUNE_GU", "MOE_TUNE_DOWN", "MOE_TUNE_WIDE"):
        assert v not in os.environ, f"{v} overrides the rules this test checks"
    from paper_2509_23638_amd.build import LIB, build
    if not os.path.exists(LIB):
        build(verbose=False)
    import paper_2509_23638_amd.binding as B
    return B


def _names(B, cfg, T=None):
    sh = B.make_shape(T if T is not None else cfg.T, cfg.H, cfg.E, cfg.k, cfg.F, cfg.S, cfg.dtype, "tiled")
    n = cfg.E + cfg.S
    return B.moe_ffn_kernel_name(sh, 0, n), B.moe_ffn_kernel_name(sh, 1, n)


def test_mixtral_decode_sizes(B):
    cfg = get_config("c2_mixtral")
    # wide experts: the persistent tiled kernel streams gate/up at every decode batch
    assert _names(B, cfg, 64) == ("ffn_tile_small_kernel<gate/up>", "ffn_tile_small_kernel<down>")
    # the down projection too, once its (active expert, 128 columns) items about fill the chip
    assert _names(B, cfg, 32) == ("ffn_tile_small_kernel<gate/up>", "ffn_tile_small_kernel<down>")
    assert _names(B, cfg, 12) == ("ffn_tile_small_kernel<gate/up>", "ffn_tile_small_kernel<down>")
    assert _names(B, cfg, 10) == ("ffn_tile_small_kernel<gate/up>", "ffn_down_splitk_kernel")
    assert _names(B, cfg, 65) == ("ffn_tile_kernel<gate/up>", "ffn_tile_kernel<down>")
    assert _names(B, cfg, 1) == ("ffn_tile_small_kernel<gate/up>", "ffn_down_splitk_kernel")
    assert _names(B, cfg, 8) == ("ffn_tile_small_kernel<gate/up>", "ffn_down_splitk_kernel")
    # from about 24 rows per expert both phases are tiled, from 96 in the eight-wave form
    assert _names(B, cfg, 256) == ("ffn_tile_kernel<gate/up>", "ffn_tile_kernel<down>")
    assert _names(B, cfg, 512) == ("ffn_wide_kernel<gate/up>", "ffn_wide_kernel<down>")


def test_fine_grained_and_prefill(B):
    # shared experts over about a hundred tokens: gate/up in 256-row blocks of the tiled
    # kernel (one pass over their weights), down in the stream kernel's 64-column form
    assert _names(B, get_config("c3_finegrained")) == (
        "ffn_tile_kernel<gate/up>", "ffn_stream_kernel<down, 64 rows>")
    c3 = get_config("c3_finegrained")
    assert _names(B, c3, 96) == ("ffn_stream_kernel<gate/up, 64 rows>", "ffn_stream_kernel<down, 64 rows>")
    assert _names(B, c3, 256) == ("ffn_tile_kernel<gate/up>", "ffn_stream_kernel<down, 64 rows>")
    assert _names(B, c3, 257) == ("ffn_wide_kernel<gate/up>", "ffn_wide_kernel<down>")
    assert _names(B, get_config("c4_dsv2lite_prefill")) == (
        "ffn_wide_kernel<gate/up>", "ffn_wide_kernel<down>")
    # many experts with a few rows each: enough workgroups without split-K
    assert _names(B, get_config("c6_qwen3_a3b")) == (
        "ffn_stream_kernel<gate/up, 64 rows>", "ffn_stream_kernel<down, halved contraction>")


def test_choice_does_not_depend_on_the_number_of_listed_experts_once_blocks_are_filled(B):
    """The streamed path calls the FFN over subsets of experts; with well-filled
    blocks every such call must land on the same kernels as the all-resident
    call (the eight-wave form is chosen from the shape alone)."""
    for name, T in (("c4_dsv2lite_prefill", None), ("c5_stack", None), ("c2_mixtral", 1),
                    ("c2_mixtral", 64), ("c2_mixtral", 256), ("c3_finegrained", None),
                    ("c6_qwen3_a3b", None)):
        cfg = get_config(name)
        sh = B.make_shape(T or cfg.T, cfg.H, cfg.E, cfg.k, cfg.F, cfg.S, cfg.dtype, "tiled")
        for phase in (0, 1):
            names = {B.moe_ffn_kernel_name(sh, phase, n) for n in (1, 2, 7, 33, cfg.E + cfg.S)}
            assert len(names) == 1, (name, names)


def test_the_small_tiled_kernel_is_chosen_by_the_token_count_alone(B):
    """At most 64 tokens: every bucket of a well-formed routing fits one 64-row
    block, which is what the small tiled kernel multiplies per item (it splits a
    larger bucket into 64-row blocks rather than cutting it)."""
    cfg = get_config("c2_mixtral")
    for T, want in ((1, "small"), (64, "small"), (65, "tile_kernel"), (128, "tile_kernel")):
        sh = B.make_shape(T, cfg.H, cfg.E, cfg.k, cfg.F, cfg.S, cfg.dtype, "tiled")
        assert want in B.moe_ffn_kernel_name(sh, 0, cfg.E)


def test_rows_of_y_are_bf16_exactly_where_the_down_projection_runs_its_prefill_form(B):
    """The block keeps Y in bf16 only at prefill sizes; the decision is the shape's."""
    import torch
    for name, T in (("c4_dsv2lite_prefill", None), ("c2_mixtral", 512), ("c2_mixtral", 64), ("c2_mixtral", 256),
                    ("c3_finegrained", None), ("c5_stack", None), ("c6_qwen3_a3b", None), ("c1_tiny", None)):
        cfg = get_config(name)
        sh = B.make_shape(T or cfg.T, cfg.H, cfg.E, cfg.k, cfg.F, cfg.S, cfg.dtype,
                          "tiled" if cfg.dtype == "bf16" else "row_major")
        wide = B.moe_ffn_kernel_name(sh, 1, cfg.E + cfg.S) == "ffn_wide_kernel<down>"
        assert (B.moe_layer_y_dtype(sh) == torch.bfloat16) == wide, name
    assert B.moe_layer_y_dtype(B.make_shape(2048, 2048, 64, 6, 1408, 2, "bf16", "tiled")) == torch.bfloat16


def test_product_build_has_no_tuning_overrides(B):
    """MOE_TUNE_* environment overrides exist only in measurement builds."""
    assert "tuning" not in B.moe_version()


def test_f32_storage_has_its_own_kernel(B):
    cfg = get_config("c1_tiny")
    sh = B.make_shape(cfg.T, cfg.H, cfg.E, cfg.k, cfg.F, cfg.S, "f32", "row_major")
    assert B.moe_ffn_kernel_name(sh, 0, cfg.E) == "ffn_f32_kernel<gate/up>"
    assert B.moe_ffn_kernel_name(sh, 1, cfg.E) == "ffn_f32_kernel<down>"
