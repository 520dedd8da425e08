"""GPU parity, element by element, at sizes the oracle finishes in seconds: every
kernel variant (group size, pixels per lane, resident / chunked / 3x3, vector and
scalar staging, MFMA and FMA inner loops), ragged tails and degenerate masks."""
import numpy as np
import pytest

import paper_2109_00170_amd as alcs
import workloads
from gpu_util import TOL, oracle_ref, rel_err, run_dense, run_sparse

pytestmark = pytest.mark.gpu


def check(L, seed, with_bias=True, **tuning):
    d = workloads.make_layer(L, seed, with_bias=with_bias)
    got, info = run_sparse(d, options=tuning)
    ref = oracle_ref(d)
    assert got.shape == ref.shape
    assert not np.isnan(got).any(), "some outputs were never written"
    err = rel_err(got, ref)
    assert err <= TOL, "%s %s: rel err %.3g" % (L.name, info, err)
    return info


def test_config1_single_pointwise_layer():
    """Config 1: 1x1, batch 1, 64->64 at 56x56, V=4, 512 of 1024 blocks kept."""
    L = workloads.config1()
    d = workloads.make_layer(L, workloads.seed_for(1, 0))
    assert d.nnzb == 512
    got, info = run_sparse(d)
    assert rel_err(got, oracle_ref(d)) <= TOL


@pytest.mark.parametrize("V", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("pv", [1, 2, 4])
def test_pointwise_resident_all_group_sizes(V, pv):
    # 3 images of 20x20 = 1200 pixels: several tiles and a ragged last tile; Cout=44 is ragged for V=8,16
    L = workloads.Layer("pw_v%d" % V, 48, 44, 20, 20, N=3, V=V, sparsity=0.6, x_dist="relu")
    info = check(L, 100 + V, pv=pv)
    assert info["mode"] == 1 and info["pv"] == pv


@pytest.mark.parametrize("V,pv", [(4, 1), (4, 2), (4, 4), (8, 1), (8, 4), (16, 2)])
def test_pointwise_streaming_kernel(V, pv):
    """Enough pixels for the persistent double-buffered kernel; 3 x 212 x 212 pixels do
    not divide evenly among the workgroups, so the last tile of every range is partial."""
    L = workloads.Layer("pw_stream_v%d" % V, 24, 40, 212, 212, N=3 * pv, V=V, sparsity=0.7, x_dist="relu")
    info = check(L, 150 + V + pv, pv=pv, path=4)
    assert info["mode"] == 4 and info["pv"] == pv


def test_pointwise_many_pixels_resident_kernel():
    L = workloads.Layer("pw_nostream", 24, 40, 212, 212, N=3, V=4, sparsity=0.7, x_dist="relu")
    info = check(L, 160)
    assert info["mode"] == 1


@pytest.mark.parametrize("V", [1, 4, 8])
def test_pointwise_odd_pixel_count_uses_scalar_staging(V):
    L = workloads.Layer("pw7x7_v%d" % V, 40, 24, 7, 7, N=5, V=V, sparsity=0.5)
    info = check(L, 200 + V)
    assert info["mode"] == 1 and info["pv"] == 1


@pytest.mark.parametrize("V", [2, 4, 16])
def test_pointwise_stride2(V):
    L = workloads.Layer("pw_s2_v%d" % V, 24, 32, 15, 13, k=1, stride=2, N=2, V=V, sparsity=0.5)
    check(L, 300 + V)


@pytest.mark.parametrize("V,kc", [(1, 16), (4, 16), (4, 40), (8, 24), (16, 64)])
def test_pointwise_chunked(V, kc):
    L = workloads.Layer("pw_chunk_v%d" % V, 100, 72, 12, 12, N=3, V=V, sparsity=0.7)
    info = check(L, 400 + V + kc, chunk_channels=kc)
    assert info["mode"] == 2 and info["chunk_channels"] == kc


@pytest.mark.parametrize("V,gs", [(4, 2), (4, 4), (8, 2), (16, 4)])
@pytest.mark.parametrize("hw", [12, 7])
def test_pointwise_several_groups_per_wavefront(V, gs, hw):
    """2 or 4 groups share a wavefront (32 or 16 pixels each); Cout=44 leaves the last
    bundle partly empty, hw=7 exercises the scalar staging path."""
    L = workloads.Layer("pw_gs%d_v%d" % (gs, V), 60, 44, hw, hw, N=5, V=V, sparsity=0.6)
    info = check(L, 430 + V + gs + hw, group_slots=gs)
    assert info["mode"] == 1 and info["group_slots"] == gs


@pytest.mark.parametrize("V,gs", [(4, 2), (4, 4), (8, 2), (8, 4), (16, 2), (16, 4)])
@pytest.mark.parametrize("hw", [12, 7])
def test_pointwise_several_groups_per_wavefront_two_pixels_per_lane(V, gs, hw):
    """The same with two pixels per lane (64 or 32 pixels per tile): an aligned pair at 12x12,
    two pixels half a tile apart at 7x7, where neighbours may lie in different images.  5
    images leave a ragged last tile, Cout=44 a partly empty last bundle."""
    L = workloads.Layer("pw_gs%d_v%d_pv2" % (gs, V), 60, 44, hw, hw, N=5, V=V, sparsity=0.6)
    info = check(L, 440 + V + gs + hw, group_slots=gs, pv=2)
    assert info["mode"] == 1 and info["group_slots"] == gs and info["pv"] == 2


@pytest.mark.parametrize("Cin,Cout,hw,N", [(512, 64, 14, 32),    # four groups per wavefront, pixel pairs: 28 of 32 pixels
                                           (512, 64, 7, 120),    # the same where pairs are half a tile apart: 24 of 32
                                           (1300, 64, 14, 15)])  # one pixel per lane: 16-pixel tiles, 12 of 16
def test_pointwise_single_round_spreads_pixels_over_all_compute_units(Cin, Cout, hw, N):
    """A launch of one round with fewer workgroups than compute units gives every workgroup
    fewer pixels than its tile holds; the option full_tiles keeps full tiles.  Both must match the oracle."""
    L = workloads.Layer("pw_narrow", Cin, Cout, hw, hw, N=N, V=4, sparsity=0.9)
    full = check(L, 480 + Cin + hw, full_tiles=1)
    spread = check(L, 480 + Cin + hw)
    assert full["mode"] == 1 and spread["mode"] == 1
    assert spread["workgroups"] > full["workgroups"], (full, spread)
    assert spread["workgroups"] <= 256


def test_pointwise_many_tiles_of_a_register_heavy_kernel_take_8_wavefronts():
    """More workgroups than compute units, tiles of which two fit a compute unit, and a kernel
    that holds more than 64 registers per lane (four groups per wavefront): 8 wavefronts per
    workgroup, so that two workgroups share a compute unit; a single round keeps 16."""
    many = workloads.Layer("pw_many_tiles", 512, 64, 28, 28, N=12, V=4, sparsity=0.9)
    info = check(many, 490)
    assert info["group_slots"] == 4 and info["workgroups"] > 256 and info["waves"] == 8, info
    few = workloads.Layer("pw_few_tiles", 512, 256, 14, 14, N=8, V=4, sparsity=0.9)
    info = check(few, 491)
    assert info["group_slots"] == 4 and info["workgroups"] <= 256 and info["waves"] == 16, info


@pytest.mark.parametrize("Cin,gs", [(512, 4), (1100, 4), (2048, 4)])
def test_pointwise_wide_inputs_pair_groups_by_default(Cin, gs):
    L = workloads.Layer("pw_wide%d" % Cin, Cin, 40, 7, 7, N=3, V=4, sparsity=0.9)
    info = check(L, 450 + gs)
    assert info["mode"] == 1 and info["group_slots"] == gs


def test_pointwise_very_wide_or_small_v_inputs_are_chunked():
    info = check(workloads.Layer("pw_wide_v1", 700, 12, 7, 7, N=3, V=1, sparsity=0.9), 456)
    assert info["mode"] == 2
    info = check(workloads.Layer("pw_wide2600", 2600, 16, 5, 5, N=2, V=4, sparsity=0.95), 457)
    assert info["mode"] == 2


def test_pointwise_fma_path_for_v4_matches_too():
    L = workloads.Layer("pw_fma", 64, 64, 16, 16, N=2, V=4, sparsity=0.5)
    info = check(L, 460, path=1)
    assert info["path"] == 1
    info = check(L, 460, path=2)
    assert info["path"] == 2


@pytest.mark.parametrize("groups", [1, 3])
def test_pointwise_group_tiles(groups):
    L = workloads.Layer("pw_gt", 64, 96, 10, 10, N=2, V=4, sparsity=0.5)
    info = check(L, 470, group_tiles=groups, waves=2)
    assert info["group_tiles"] == groups


@pytest.mark.parametrize("V", [1, 4, 8])
@pytest.mark.parametrize("stride", [1, 2])
def test_conv3x3(V, stride):
    # 19x17: tiles of 8x8 with ragged right/bottom edges; 40 channels = 2 chunks of 32
    L = workloads.Layer("c3_v%d_s%d" % (V, stride), 40, 36, 19, 17, k=3, stride=stride, N=2, V=V,
                        sparsity=0.7, w_std=0.05)
    info = check(L, 500 + V + stride)
    assert info["mode"] == 3


@pytest.mark.parametrize("V", [1, 2, 4, 16])
@pytest.mark.parametrize("stride", [1, 2])
@pytest.mark.parametrize("tile_width", [8, 16, 32])
def test_conv3x3_tile_shapes(V, stride, tile_width):
    # 37 columns: one full 32-wide tile and a ragged one; 21 rows: ragged for every tile
    # height; 70 channels = 3 chunks, the last one short; ragged last group for V = 16
    L = workloads.Layer("c3_tw%d_v%d_s%d" % (tile_width, V, stride), 70, 40, 21, 37, k=3, stride=stride,
                        N=2, V=V, sparsity=0.75, w_std=0.05)
    info = check(L, 540 + V + 3 * stride + tile_width, tile_width=tile_width)
    assert info["mode"] == 3 and info["tile_width"] == tile_width


@pytest.mark.parametrize("V", [4, 8])
@pytest.mark.parametrize("tile_width", [8, 16, 32])
@pytest.mark.parametrize("ug", [2, 4])
def test_conv3x3_two_pixels_per_lane(V, tile_width, ug):
    """Stride 1, tiles of twice the height, a lane owns two pixels a fixed number of rows apart:
    21 rows are ragged for 16-, 8- and 4-row tiles, 37 columns for every width; 70 channels =
    3 chunks, the last one short."""
    L = workloads.Layer("c3_tall_tw%d_v%d" % (tile_width, V), 70, 40, 21, 37, k=3, stride=1, N=2, V=V,
                        sparsity=0.75, w_std=0.05)
    info = check(L, 545 + V + tile_width + ug, tile_width=tile_width, pv=2, groups_per_wave=ug)
    assert info["mode"] == 3 and info["tile_width"] == tile_width and info["pv"] == 2


def test_conv3x3_two_pixels_per_lane_small_and_odd_images():
    for hw, seed in ((7, 1), (5, 2), (1, 3), (14, 4)):
        L = workloads.Layer("c3_tall_%d" % hw, 24, 16, hw, hw, k=3, stride=1, N=3, V=4, sparsity=0.5)
        info = check(L, 548 + seed, pv=2)
        assert info["pv"] == 2
    # stride 2 and V = 16 keep one pixel per lane
    L = workloads.Layer("c3_tall_s2", 24, 16, 9, 9, k=3, stride=2, N=2, V=4, sparsity=0.5)
    assert check(L, 553, pv=2)["pv"] == 1
    L = workloads.Layer("c3_tall_v16", 24, 32, 9, 9, k=3, stride=1, N=2, V=16, sparsity=0.5)
    assert check(L, 554, pv=2)["pv"] == 1


@pytest.mark.parametrize("tile_width", [8, 16, 32])
def test_conv3x3_tile_shapes_few_waves_use_position_loop(tile_width):
    L = workloads.Layer("c3_tw%d_small_wg" % tile_width, 16, 16, 11, 35, k=3, stride=2, N=1, V=4, sparsity=0.5)
    check(L, 560 + tile_width, waves=2, tile_width=tile_width)


def test_conv3x3_tap_shared_pattern_and_many_groups():
    L = workloads.Layer("c3_shared", 64, 200, 14, 14, k=3, stride=1, N=2, V=4, sparsity=0.8,
                        w_std=0.05, tap_shared=True)
    check(L, 520)


def test_conv3x3_few_waves_uses_position_loop():
    L = workloads.Layer("c3_small_wg", 16, 16, 9, 9, k=3, stride=2, N=1, V=4, sparsity=0.5)
    check(L, 530, waves=2)


def test_degenerate_masks():
    import torch
    L = workloads.Layer("deg", 32, 16, 8, 8, N=2, V=4, sparsity=0.5)
    d = workloads.make_layer(L, 600, with_bias=True)
    # everything dropped: output is the bias, exactly
    d.mask[:] = 0
    got, _ = run_sparse(d)
    assert np.array_equal(got, np.broadcast_to(d.bias[None, :, None, None], got.shape))
    # everything kept equals the dense conv of the oracle
    d.mask[:] = 1
    got, _ = run_sparse(d)
    assert rel_err(got, oracle_ref(d)) <= TOL
    # one group empty, one full
    d.mask[:] = 0
    d.mask[1] = 1
    got, _ = run_sparse(d)
    assert rel_err(got, oracle_ref(d)) <= TOL
    assert np.array_equal(got[:, :4], np.broadcast_to(d.bias[None, :4, None, None], got[:, :4].shape))
    del torch


def test_identity_input_reads_back_weights_exactly():
    """1x1 with X one-hot per channel: every sum has one term, so Y is the pruned
    weight matrix bit for bit - pins the column indexing through the compute path."""
    V, Cin, Cout = 4, 64, 40
    L = workloads.Layer("ident", Cin, Cout, 8, 8, N=1, V=V, sparsity=0.5)
    d = workloads.make_layer(L, 700)
    d.X[:] = np.eye(Cin, dtype=np.float32).reshape(1, Cin, 8, 8)
    got, _ = run_sparse(d)
    keep = np.repeat(d.mask.reshape(L.G, Cin), V, axis=0)[:Cout].astype(bool)
    expect = np.where(keep, d.W.reshape(Cout, Cin), np.float32(0))
    assert got.reshape(Cout, Cin).tobytes() == expect.tobytes()


def test_impulse_3x3_exact():
    L = workloads.Layer("imp", 1, 4, 9, 9, k=3, stride=1, N=1, V=4, sparsity=0.0)
    d = workloads.make_layer(L, 710)
    d.X[:] = 0
    d.X[0, 0, 4, 5] = 1.0
    got, _ = run_sparse(d)
    ref = oracle_ref(d)
    assert got.tobytes() == ref.tobytes()


@pytest.mark.parametrize("k,stride,Cout,Cin,HW,N", [(1, 1, 64, 64, 56, 1), (1, 1, 200, 70, 14, 3),
                                                    (1, 1, 40, 33, 7, 5), (1, 2, 24, 20, 9, 2),
                                                    (3, 1, 36, 20, 12, 2), (3, 2, 130, 17, 11, 2)])
def test_dense_conv(k, stride, Cout, Cin, HW, N):
    L = workloads.Layer("dense", Cin, Cout, HW, HW + (0 if k == 1 and stride == 1 and HW % 2 == 0 else 1),
                        k=k, stride=stride, N=N, V=4, sparsity=0.0, w_std=0.05, mask_kind="none")
    d = workloads.make_layer(L, 800 + Cout, with_bias=True)
    got = run_dense(d)
    ref = oracle_ref(d)
    assert not np.isnan(got).any()
    assert rel_err(got, ref) <= TOL


def test_sparse_at_sparsity_zero_equals_dense():
    L = workloads.Layer("s0", 96, 64, 14, 14, N=2, V=4, sparsity=0.0)
    d = workloads.make_layer(L, 900, with_bias=True)
    a, _ = run_sparse(d)
    b = run_dense(d)
    assert rel_err(a, b) <= TOL


@pytest.mark.parametrize("Cin,Cout,H,W,N", [
    (64, 72, 14, 14, 9),     # 28-pixel tiles that tile the image; ordinary stores (planes off the line grid)
    (40, 72, 8, 8, 21),      # 32-pixel tiles, planes on the line grid: streaming stores
    (56, 40, 6, 10, 11),     # 60 pixels per image: tiles straddle images, ragged last tile
    (64, 520, 14, 14, 5),    # 33 bundles: two group tiles
    (48, 24, 2, 2, 50),      # 4 pixels per image, 8 images per tile
    (512, 64, 14, 14, 40),   # 512 input channels (the widest the kernel takes), 280 tiles on 256 workgroups
])
def test_pointwise_pipelined_persistent(Cin, Cout, H, W, N):
    """The persistent double-buffered kernel of the many-tile regime (four groups per wavefront,
    weights resident in registers), forced onto small layers: one, two and more tiles per
    workgroup, with and without bias."""
    L = workloads.Layer("pipe_%d_%d" % (Cin, Cout), Cin, Cout, H, W, k=1, stride=1, N=N, V=4,
                        sparsity=0.6 if Cin <= 64 else 0.93, w_std=0.2, x_dist="uniform")
    for with_bias in (False, True):
        info = check(L, 77 + Cin + Cout, with_bias=with_bias, group_slots=4, path=5)
        assert info["mode"] == 5 and info["group_slots"] == 4, info


@pytest.mark.parametrize("Cin,Cout,sparsity,N", [(512, 136, 0.87, 40), (200, 72, 0.62, 12), (160, 40, 0.55, 30)])
def test_pointwise_pipelined_persistent_long_segments(Cin, Cout, sparsity, N):
    """Segments of 65 to 96 columns: one bundle per wavefront, the runs beyond the fourth through
    two temporaries inside the multiply."""
    L = workloads.Layer("pipe_long_%d" % Cin, Cin, Cout, 14, 14, k=1, stride=1, N=N, V=4, sparsity=sparsity, w_std=0.2,
                        x_dist="uniform")
    d = workloads.make_layer(L, 91 + Cin)
    longest = int(d.mask.reshape(L.G, -1).sum(axis=1).max())
    assert 64 < longest <= 96, longest
    info = check(L, 91 + Cin, with_bias=True, group_slots=4, path=5)
    assert info["mode"] == 5 and info["group_slots"] == 4, info
