"""Address arithmetic of the depthwise stage of the fused MobileNet block (stage_dw_mode in
csrc/alcs_sparse.hip, offsets as in csrc/alcs_dw_taps.h), walked on the CPU for every thread, tap and
channel of a launch: every address the kept schedule - two channels in flight under the guard
`c + rpp < Cin` - forms lies inside X and every (channel, tile position) is produced exactly once.

The same walk also shows what a four-channel schedule does under that two-channel guard: its third
and fourth load reach channels beyond Cin, which in the last image is memory behind X.  A variant
with four channels in flight once faulted on the GPU and was taken out; its source was not kept, so
this is the probable cause, not a proven one - the walk pins the arithmetic the kernel relies on and
the failure a longer pipeline under the old guard would have.
"""
import numpy as np
import pytest


def walk(N, Cin, H, W, stride, TP, nt, loads, guard_loads):
    """Returns (addresses out of bounds, cells produced, cells expected, duplicates)."""
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    P, Pin = Ho * Wo, H * W
    NP, total = N * P, N * Cin * Pin
    span = min(nt, TP)
    rpp = nt // span
    bad = 0
    produced = {}
    for q0 in range(0, NP, TP):
        q_end = min(NP, q0 + TP)
        for wave in range(nt // 64):
            tid = np.arange(wave * 64, wave * 64 + 64)
            r0 = tid // span
            if TP >= 64:
                r0 = np.full(64, r0[0])                      # readfirstlane: the span is a multiple of 64
            act = r0 < rpp
            if not act.any():
                continue
            e = tid - r0 * span
            while (e[act] < TP).any():
                live = act & (e < TP)
                q = q0 + e
                valid = q < q_end
                n = np.where(valid, q // P, 0)
                po = np.where(valid, q - n * P, 0)
                ho, wo = po // Wo, po % Wo
                n0 = int(n[np.nonzero(live)[0][0]])          # the wavefront's first active lane
                rl = np.zeros(64, np.int64) if TP >= 64 else r0.astype(np.int64)
                delta = np.where(valid, ((n - n0) * Cin + rl) * Pin, rl * Pin).astype(np.int64)
                offs = []
                for r in range(3):
                    for t in range(3):
                        hc = np.clip(ho * stride - 1 + r, 0, H - 1)
                        wc = np.clip(wo * stride - 1 + t, 0, W - 1)
                        # 32-bit byte offsets, as the kernel forms them
                        offs.append((((delta + hc * W + wc) & 0xFFFFFFFF) * 4) & 0xFFFFFFFF)
                for lane in np.nonzero(live)[0]:
                    c = int(r0[lane])
                    chans = []
                    while TP >= 64 and c + (guard_loads - 1) * rpp < Cin:
                        chans += [c + u * rpp for u in range(loads)]
                        c += loads * rpp
                    while c < Cin:
                        chans.append(c)
                        c += rpp
                    for ch in chans:
                        base = ((n0 * Cin + ch - int(rl[lane])) * Pin) * 4
                        for o in offs:
                            a = base + int(o[lane])
                            if a < 0 or a + 4 > total * 4:
                                bad += 1
                        if ch < Cin:
                            key = (ch, q0, int(e[lane]))
                            produced[key] = produced.get(key, 0) + 1
                e = e + span
    ntiles = (NP + TP - 1) // TP
    dup = sum(1 for v in produced.values() if v != 1)
    return bad, len(produced), Cin * ntiles * TP, dup


# (N, Cin, H, W, stride, TP, threads): the launches of the GPU tests of the block, among them the
# shape on which the four-channel variant faulted (8 output channels per group, 4 pixels per lane:
# 256-pixel tiles on 1024 threads, 40 channels, 17 x 16 images)
LAUNCHES = [(3, 40, 17, 16, 1, 256, 1024), (3, 40, 17, 16, 1, 256, 320), (2, 10, 20, 20, 1, 256, 64),
            (5, 40, 9, 7, 1, 32, 512), (4, 64, 14, 14, 1, 32, 1024), (9, 70, 14, 14, 2, 16, 1024),
            (3, 33, 9, 20, 2, 64, 256), (1, 3, 1, 1, 1, 64, 64), (2, 130, 33, 2, 1, 128, 512)]


@pytest.mark.parametrize("launch", LAUNCHES)
def test_two_channels_in_flight_stay_inside_the_input(launch):
    bad, cells, expected, dup = walk(*launch, loads=2, guard_loads=2)
    assert bad == 0
    assert cells == expected and dup == 0


def test_four_channels_under_the_two_channel_guard_read_behind_the_input():
    # the launch that faulted: channels 40 and 44 of the last image do not exist
    bad, _, _, _ = walk(3, 40, 17, 16, 1, 256, 1024, loads=4, guard_loads=2)
    assert bad > 0
    # with a guard that covers all four loads the same schedule is in bounds and complete
    bad, cells, expected, dup = walk(3, 40, 17, 16, 1, 256, 1024, loads=4, guard_loads=4)
    assert bad == 0 and cells == expected and dup == 0
