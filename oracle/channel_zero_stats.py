"""How often would skipping along the channel (K) dimension of a convolution fire?

TEST / EVIDENCE INFRASTRUCTURE: calls only the CPU oracle and the seeded input generators, never
the HIP library.  It writes the summary committed as profiles/unet_depth_channel_zero_statistics.md:

    python oracle/channel_zero_stats.py > profiles/unet_depth_channel_zero_statistics.md

The paper's mask element covers an h x w section of ONE channel ("Implementation of Increment
Layers"), so its convolution can skip the filter applications of a section of a single channel
that is entirely zero ("Convolution on Sparse Inputs").  A matrix-core kernel contracts a tile
against channel groups: the smallest unit it could skip is one 8 x 8 tile of sites x 8 channels
(fp32 operands) or x 16 channels (bf16 operands).  For every node of the UNet depth network that
feeds a convolution, after a few steps of the workload-3 stream, this script counts, over the
tiles that hold at least one active site:
  * the fraction of increment elements at active sites that are zero,
  * the fraction of (tile, single channel) sections that are entirely zero (the paper's unit),
  * the fraction of (tile, 8-channel group), (tile, 16-channel group) and (tile, 32-channel group)
    sections that are entirely zero (what a matrix-core kernel could skip),
in the lossless mode, with a sparsification layer (t_p = 0.1) ahead of every convolution, and with
those layers on the stream with small-valued increments.
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle.oracle import Oracle, SET_ACTIVE  # noqa: E402
from paper_2303_04670_amd import workloads as wl  # noqa: E402

H, W, STEPS, STEPS_SMALL = 256, 352, 4, 24


def stats(net, frames, title):
    ora = Oracle(net)
    ora.reset(frames[0])
    for f in frames[1:]:
        ora.step_frame(f)
    consumers = {nd.in0 for nd in net.nodes if nd.op == wl.OP_CONV2D}
    print(f"\n## {title} (state after {len(frames) - 1} steps)\n")
    print("| node | op | C | H x W | active sites | zero elements at active sites | all-zero (tile, 1 channel) | "
          "(tile, 8 ch) | (tile, 16 ch) | (tile, 32 ch) |")
    print("|---|---|---|---|---|---|---|---|---|---|")
    tot = {8: [0, 0], 16: [0, 0], 32: [0, 0], 1: [0, 0]}
    for i, nd in enumerate(net.nodes):
        if i not in consumers:
            continue
        c, h, w = ora.shape(i)
        if c < 32:
            continue
        dy = ora.dy(i)
        act = ora.mask(i, SET_ACTIVE).astype(bool)
        if act.sum() == 0:
            print(f"| {i} | {nd.op} | {c} | {h} x {w} | 0 | - | - | - | - | - |")
            continue
        zero_el = float((dy[act] == 0).mean())
        h8, w8 = (h + 7) // 8 * 8, (w + 7) // 8 * 8
        pad = np.zeros((h8, w8, c))
        pad[:h, :w] = dy
        t = np.abs(pad).reshape(h8 // 8, 8, w8 // 8, 8, c).max(axis=(1, 3))   # tiles x channels: largest magnitude
        tile_on = t.max(axis=2) > 0
        cells = []
        for g in (1, 8, 16, 32):
            blk = t.reshape(t.shape[0], t.shape[1], c // g, g).max(axis=3) == 0
            cells.append(float(blk[tile_on].mean()))
            tot[g][0] += int(blk[tile_on].sum())
            tot[g][1] += int(blk[tile_on].size)
        print(f"| {i} | {nd.op} | {c} | {h} x {w} | {int(act.sum())} | {zero_el:.3f} | {cells[0]:.4f} | {cells[1]:.4f} | "
              f"{cells[2]:.4f} | {cells[3]:.4f} |")
    print(f"\nAll listed nodes together: all-zero (tile, 1 channel) {tot[1][0]} of {tot[1][1]}; (tile, 8 channels) "
          f"{tot[8][0]} of {tot[8][1]}; (tile, 16 channels) {tot[16][0]} of {tot[16][1]}; (tile, 32 channels) "
          f"{tot[32][0]} of {tot[32][1]}.")


def main():
    print("# Channel-dimension sparsity of the increments (CPU oracle), UNet depth net 5x256x352\n")
    print("Written by `python oracle/channel_zero_stats.py` (oracle and seeded generators only).  op codes: 0 conv, 1 add, 3 up-sampling, 8 sparsification layer.  Only nodes that "
          "feed a convolution and have at least 32 channels are listed.")
    frames = list(wl.stream_voxel(1003, H, W, STEPS, 0.02))
    stats(wl.net_unet_depth(1003, h=H, w=W), frames, "Lossless, workload-3 stream (2 % changed pixels)")
    net = wl.net_unet_depth(1003, h=H, w=W, sparsify=True)
    net.sparsify_tp = 0.1
    stats(net, frames, "Sparsification layer ahead of every convolution, t_p = 0.1, workload-3 stream")
    # (the residuals of the sparsification layers take some twenty steps to fill up on this stream)
    frames = list(wl.stream_voxel_drifting_background(1003, H, W, STEPS_SMALL, 0.02))
    for tp in (0.1, 0.3):
        net = wl.net_unet_depth(1003, h=H, w=W, sparsify=True, sparsify_input=True)
        net.sparsify_tp = tp
        stats(net, frames, f"Sparsification layers (also on the input), t_p = {tp}, stream with small-valued increments")


if __name__ == "__main__":
    main()
