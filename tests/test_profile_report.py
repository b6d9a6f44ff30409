"""Host-side checks of the measurement plumbing: the profiler-name mapping of the report generator and
the parser that bench.py applies to the committed HBM-traffic summary."""
import os
import re
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

from paper_2108_09413_amd import profile_report  # noqa: E402


def test_profiler_names_map_to_the_librarys_instance_names():
    f = profile_report.library_name
    assert f("void isr::conv_dma_kernel<256, 256, 128, 2, 0, 1, true, 64, 64, true>(isr::ConvParams)") == \
        "conv_dma_kernel<256, 256, 128, 2, 0, 1, 64x64>"
    assert f("void isr::conv_dma_kernel<128, 128, 64, 2, 2, 3, true, 64, 64, false>(isr::ConvParams)") == \
        "conv_dma_kernel<128, 128, 64, 2, 2, 3, 64x64>"
    assert f("void isr::conv_dma_kernel<256, 256, 128, 2, 0, 1, false, 128, 64>(isr::ConvParams)") == \
        "conv_dma_kernel<256, 256, 128, 2, 0, 1, 128x64>"
    assert f("void isr::(anonymous namespace)::conv_patch_kernel<128, 64, 2, false, true>(isr::ConvParams)") == \
        "conv_patch_kernel<128, 256, 64>"
    assert f("void isr::(anonymous namespace)::expand_reduce_kernel<true>(isr::XrParams)") == "expand_reduce_kernel<128, 512, 128>"
    assert f("void isr::(anonymous namespace)::expand_reduce1024_kernel<true>(isr::XrParams)") == "expand_reduce_kernel<256, 1024, 256>"
    assert f("void isr::(anonymous namespace)::expand_reduce256_kernel<true>(isr::XrParams)") == "expand_reduce_kernel<128, 512, 256>"
    assert f("void isr::(anonymous namespace)::proj_expand_reduce_kernel<false>(isr::XrParams)") == \
        "proj_expand_reduce_kernel<256, 128, 512, 128>"
    assert f("void isr::(anonymous namespace)::bottleneck_kernel<2, true>(isr::BneckParams)") == \
        "bottleneck_kernel<block + projection, true>"
    assert f("void isr::(anonymous namespace)::fconv_kernel<2, 2, 2, 2>(isr::FConvParams)") == "fconv_kernel<128 x 128>"
    assert f("isr::(anonymous namespace)::stem_pool_kernel(isr::StemPoolParams)") == "stem_pool_kernel (+noise)"
    assert f("isr::gap_kernel(isr::GapParams)") == "gap_kernel"
    assert profile_report.is_conv("fconv_kernel<64 x 128>") and not profile_report.is_conv("gap_kernel")


def test_committed_traffic_summary_parses_and_names_instances_as_the_library_does():
    import bench
    path = os.path.join(ROOT, "profiles", "resnet50_certify_hbm_traffic.md")
    txt = open(path).read()
    assert re.search(r"sources_sha256: [0-9a-f]{64}", txt)
    names = re.findall(r"^kernel_bytes_per_full_chunk_launch: `([^`]+)` dispatches=\d+ fetch=\d+ write=\d+$", txt, re.M)
    assert len(names) >= 8 and re.search(r"conv_hbm_bytes_per_inference: fetch=\d+ write=\d+", txt)
    # instance names carry no profiler-only template arguments (tie-free flags)
    assert all(not re.search(r"true|false", n) or n.startswith("bottleneck_kernel") for n in names), names
    assert bench.kernel_sources_sha256() == profile_report.sources_sha256()
    traffic, src = bench.offline_traffic()
    if traffic is not None:     # the summary belongs to these sources: every line was read
        assert set(names) == set(traffic["per_kernel"]) and traffic["conv_per_inference"] > 10_000_000
    else:
        assert "other kernel sources" in src
