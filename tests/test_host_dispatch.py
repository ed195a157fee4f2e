"""CPU-only checks of the host-side planning: which kernel variant every layer of the benchmark's
ResNet-50 set is sent to, and that the workspace queries are consistent with each other."""
import pytest

import paper_2109_12191_amd as dp
from workloads import get_workload


@pytest.fixture(scope="module")
def wl():
    dp.load_library()
    return get_workload("resnet50")


def test_resnet50_layers_go_to_the_expected_kernels(wl):
    per_example, weighted = {}, {}
    for l in wl.layers:
        d = dp.make_desc(l, wl.n, wl.dtype)
        per_example[l.name] = dp.dp_kernel_variant(d, dp.DP_WS_PER_EXAMPLE_GRAD)
        weighted[l.name] = dp.dp_kernel_variant(d, dp.DP_WS_RECOMPUTE)
    # every 3x3 stride-1 conv runs in the raw-row kernel, named for its row width
    for name, width in (("s1b1.c2", 56), ("s2b2.c2", 28), ("s3b2.c2", 14)):
        assert per_example[name] == f"conv3x3_rows<bf16,w{width},per_example>"
        assert weighted[name] == f"conv3x3_rows<bf16,w{width},weighted>"
    assert weighted["s4b2.c2"] == "conv3x3_rows<bf16,w7,weighted>"
    # the strided 3x3 convs too (per-example calls only)
    assert per_example["s3b1.c2"] == "conv3x3_rows<bf16,w14,s2,per_example>"
    assert per_example["s2b1.c2"] == "conv3x3_rows<bf16,w28,s2,per_example>"
    # norm-only calls on 7x7 maps take the Gram route (3x3 convs included); their materialising calls do not
    assert per_example["s4b1.c2"] == "conv_gram_norm<bf16>" and per_example["s4b2.c2"] == "conv_gram_norm<bf16>"
    assert weighted["s2b1.c2"].startswith("conv_contract<bf16,")
    assert weighted["s4b1.c2"].startswith("conv_contract<bf16,")
    # 1x1 convs: general kernel; the classifier: the dense kernels
    assert per_example["s3b2.c3"] == "conv_contract<bf16,256x256rows,per_example>"  # 256 -> 1024 on 14x14: whole rows in blocks of 32
    from workloads import conv
    d = dp.make_desc(conv(256, 256, 1, 1, 10), 64, "bf16")
    assert dp.dp_kernel_variant(d, dp.DP_WS_PER_EXAMPLE_GRAD) == "conv_contract<bf16,256x128,per_example>"   # 10x10: chunked K
    d = dp.make_desc([l for l in wl.layers if l.name == "s2b2.c3"][0], wl.n, wl.dtype)
    assert dp.dp_kernel_variant(d, dp.DP_WS_PER_EXAMPLE_GRAD | dp.DP_VARIANT_SHARED) == \
        "conv_contract<bf16,128x128,per_example>"                                          # 28x28: K too long for the wide tile
    # norm-only calls of the 1x1 convs on 7x7 maps take the Gram route
    for name in ("s4b1.c3", "s4b2.c1", "s4b2.c3", "s4b3.c1", "s4b3.c3"):
        assert per_example[name] == "conv_gram_norm<bf16>", name
    assert per_example["s1b1.c1"] == "conv_contract<bf16,64x64,per_example>"
    assert per_example["fc"] == "dense<bf16>"
    assert sum(v.startswith("conv3x3_rows") for v in per_example.values()) == 13


def test_the_first_convolution_has_a_kernel_of_its_own_where_its_shape_allows(wl):
    from workloads import Layer, conv
    stem = "conv_stem7x7<bf16,per_example>"
    d = dp.make_desc(wl.layers[0], wl.n, wl.dtype)
    assert wl.layers[0].name == "conv1" and dp.dp_kernel_variant(d, dp.DP_WS_PER_EXAMPLE_GRAD) == stem
    assert dp.dp_kernel_variant(d, dp.DP_WS_PER_EXAMPLE_GRAD | dp.DP_VARIANT_SHARED | dp.DP_VARIANT_MATERIALISE) == stem
    assert dp.dp_norm_partial_count(d, True) == dp.dp_norm_partial_count(d, False) == 40
    # partial norms + one 64 x 160 block per range of output rows (eight ranges of 14 rows at 32 examples)
    assert dp.dp_workspace_bytes(d, dp.DP_WS_PER_EXAMPLE_GRAD) == 32 * 40 * 4 + 32 * 8 * 64 * 160 * 4
    # the clip-weighted form, fp32 inputs, a bias, odd images, other channel counts and widths that are no multiple
    # of 16 stay in the general kernel
    assert not dp.dp_kernel_variant(d, dp.DP_WS_RECOMPUTE).startswith("conv_stem")
    others = [(conv(3, 64, 7, 2, 224), "f32"), (conv(3, 64, 7, 2, 224, bias=True), "bf16"), (conv(3, 64, 7, 2, 225), "bf16"),
              (conv(3, 32, 7, 2, 224), "bf16"), (conv(4, 64, 7, 2, 224), "bf16"), (conv(3, 64, 7, 2, 24), "bf16"),
              (Layer("conv", 3, 64, 224, 224, 7, 7, 2, 2, False), "bf16"), (conv(3, 64, 7, 1, 32), "bf16")]
    for layer, dtype in others:
        name = dp.dp_kernel_variant(dp.make_desc(layer, 4, dtype), dp.DP_WS_PER_EXAMPLE_GRAD)
        assert name.startswith("conv_contract<"), (layer, dtype, name)
    # one to three input channels and any even image whose output width is a multiple of 16 do
    for layer in (conv(1, 64, 7, 2, 32), conv(2, 64, 7, 2, 64), Layer("conv", 3, 64, 38, 96, 7, 7, 2, 3, False)):
        assert dp.dp_kernel_variant(dp.make_desc(layer, 4, "bf16"), dp.DP_WS_PER_EXAMPLE_GRAD) == stem


def test_workspace_queries_are_consistent(wl):
    total = 0
    for l in wl.layers:
        d = dp.make_desc(l, wl.n, wl.dtype)
        for use in (dp.DP_WS_PER_EXAMPLE_GRAD, dp.DP_WS_RECOMPUTE):
            b = dp.dp_workspace_bytes(d, use)
            assert 0 <= b < 256 << 20, (l.name, use, b)
            assert b % 4 == 0
        for mat in (False, True):
            c = dp.dp_norm_partial_count(d, mat)
            assert 1 <= c <= 4096
            # the partial norms [n, count] sit at the start of the per-example workspace
            assert dp.dp_workspace_bytes(d, dp.DP_WS_PER_EXAMPLE_GRAD) >= 4 * wl.n * c, l.name
        total += dp.dp_workspace_bytes(d, dp.DP_WS_PER_EXAMPLE_GRAD)
    assert total < 2 << 30           # all 54 per-layer workspaces together stay small next to 288 GB


def test_descriptor_counts_match_the_layer_set(wl):
    assert sum(dp.dp_weight_count(dp.make_desc(l, wl.n, wl.dtype)) + dp.dp_bias_count(dp.make_desc(l, wl.n, wl.dtype))
               for l in wl.layers) == 25_503_912
