"""The bandwidth model against the numbers the paper's section 6 states, and
against pipelines small enough to work out by hand.  No GPU needed."""
import pytest

from paper_1705_01626_amd import cdma_model as m

PCIE3, LEFTOVER, CAP = 16.0, 236.0, 200.0     # GB/s: link, 336 - 100 left over, conservative cap


def test_average_compressor_bandwidth_of_the_paper():
    """Link bandwidth x the network-wide ratio of 2.6: about 41 GB/s on average.
    (Section 6 prints 41.3 GB/s for "16 x 2.6"; the product is 41.6, so the paper's
    figure comes from a ratio of 2.58 before rounding.  Both are checked.)"""
    assert m.comp_bw(2.6, PCIE3) == pytest.approx(41.6)
    assert m.comp_bw(41.3 / 16.0, PCIE3) == pytest.approx(41.3)
    assert round(41.3 / 16.0, 1) == 2.6
    assert m.comp_bw(2.6, PCIE3) < LEFTOVER


def test_only_layers_beyond_the_leftover_bandwidth_slow_down():
    # the best layer of the paper compresses 13.8x: 220.8 GB/s, inside 236 but above the 200 cap
    assert m.comp_bw(13.8, PCIE3) == pytest.approx(220.8)
    assert m.slowdown(13.8, PCIE3, LEFTOVER) == 1.0
    assert m.slowdown(13.8, PCIE3, CAP) == pytest.approx(220.8 / 200.0)
    assert m.slowdown(2.6, PCIE3, CAP) == 1.0
    # a 32x layer (all zeros) would need 512 GB/s
    assert m.slowdown(32.0, PCIE3, CAP) == pytest.approx(2.56)


def test_transfer_time_is_the_slower_of_link_and_memory():
    b = 1.0e9
    for ratio in (1.0, 2.6, 13.8, 32.0):
        t = m.transfer_seconds(b, ratio, PCIE3, CAP)
        assert t == pytest.approx(max(b / ratio / 16e9, b / 200e9))
    layers = [{"bytes": 1e9, "ratio": 2.0}, {"bytes": 2e9, "ratio": 32.0}]
    assert m.offload_seconds(layers, PCIE3, CAP) == pytest.approx(0.5e9 / 16e9 + 2e9 / 200e9)


def test_two_stream_pipeline_by_hand():
    # copies dominate: first compress, then the copies back to back
    assert m.two_stream_pipeline_seconds([1, 1, 1], [5, 5, 5]) == pytest.approx(1 + 15)
    # compression dominates: the last copy follows the last compress
    assert m.two_stream_pipeline_seconds([5, 5, 5], [1, 1, 1]) == pytest.approx(15 + 1)
    # mixed: c = 2,2 ; x = 3,1 -> copy0 2..5, compress1 done at 4, copy1 5..6
    assert m.two_stream_pipeline_seconds([2, 2], [3, 1]) == pytest.approx(6)
    # host gap per tensor sits on the compute stream
    assert m.two_stream_pipeline_seconds([1, 1], [0.5, 0.5], host_gap_s=1) == pytest.approx(4.5)
    assert m.two_stream_pipeline_seconds([], []) == 0.0


def test_predict_reports_link_bound_case():
    layers = [{"bytes": 800e6, "compressed_bytes": 400e6, "compress_s": 250e-6},
              {"bytes": 400e6, "compressed_bytes": 100e6, "compress_s": 120e-6}]
    p = m.predict(layers, link_gbps=50.0)
    assert p["link_bound_s"] == pytest.approx(500e6 / 50e9)
    assert p["offload_s"] == pytest.approx(250e-6 + 500e6 / 50e9)       # copies never wait again
    assert p["uncompressed_s"] == pytest.approx(1200e6 / 50e9)
    assert p["speedup"] == pytest.approx(p["uncompressed_s"] / p["offload_s"])
    assert p["max_comp_bw_needed_gbps"] == pytest.approx(4 * 50.0)
    assert p["min_encoder_read_gbps"] == pytest.approx(800e6 / 250e-6 / 1e9)
    assert p["layers_that_starve_the_link"] == 0
