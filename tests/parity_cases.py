"""The parameter sets of the GPU parity tests, kept apart from the tests themselves so that a CPU-only
test (test_variant_coverage.py) can ask the library which kernel variant each of them selects and
check that every variant the library can select is run by some GPU test."""
import numpy as np

import oracle


def P(n, c, h, w, k, kh, kw, sh=1, sw=1, ph=0, pw=0, dh=1, dw=1, g=1, bias=1):
    return dict(n=n, c=c, h=h, w=w, num_output=k, kernel_h=kh, kernel_w=kw, stride_h=sh, stride_w=sw, pad_h=ph,
                pad_w=pw, dilation_h=dh, dilation_w=dw, group=g, bias_term=bias)


# Shapes chosen to span several tiles in every dimension with ragged tails, and to hit every
# parameter: stride (incl. non-divisible), pad (incl. >= kernel extent), dilation, group,
# non-square everything, 1x1, full-size kernel, single channel.
SWEEP = [
    P(3, 5, 17, 19, 7, 3, 3),
    P(2, 3, 9, 11, 4, 1, 1),
    P(4, 6, 13, 13, 9, 13, 13),                            # kernel = input: inner product
    P(3, 4, 23, 17, 10, 3, 5, 2, 3, 1, 2),                  # non-square stride/pad/kernel
    P(2, 8, 15, 15, 12, 3, 3, 1, 1, 1, 1, 2, 2),            # dilation 2
    P(2, 4, 21, 18, 6, 3, 2, 2, 1, 2, 0, 3, 2),             # stride + dilation mix
    P(3, 6, 12, 14, 9, 3, 3, 2, 2, 1, 1, 2, 2, 3),          # groups + stride + dilation (gcd != 1)
    P(2, 2, 6, 6, 3, 3, 3, 1, 1, 3, 4),                     # pad >= kernel extent
    P(5, 1, 28, 28, 20, 5, 5),                              # layer 1.a at a small batch
    P(2, 3, 51, 51, 96, 11, 11, 4, 4),                      # 5.a-like: 96 rows, stride 4
    P(3, 16, 14, 14, 130, 5, 5, 1, 1, 2, 2, 1, 1, 2),       # 5.b-like: grouped, 65 rows per group
    P(2, 40, 13, 13, 384, 3, 3, 1, 1, 1, 1),                # 5.c-like: three 128-row tiles
    P(2, 96, 9, 9, 8, 3, 3, 1, 1, 1, 1, 1, 1, 2),           # 48 backward rows per group (16-wide MFMA tile)
    P(7, 3, 32, 32, 32, 5, 5, 1, 1, 2, 2),                  # layer 4.a at a small batch
    P(2, 4, 40, 36, 32, 8, 8, 4, 4),                        # layer 3.a-like
    P(3, 32, 20, 20, 64, 4, 4, 2, 2),                       # layer 3.b-like
    P(1, 1, 5, 7, 1, 2, 3, 3, 2, 0, 1),                     # tiny, stride > kernel
    P(2, 3, 10, 10, 5, 3, 3, 3, 3, 0, 0, 1, 1, 1, 0),       # no bias, stride leaves unread rows
    P(1, 200, 7, 7, 50, 3, 3, 1, 1, 1, 1),                  # long reduction, 50 rows (split reduction)
    P(3, 5, 30, 27, 12, 7, 7, 2, 2, 3, 3),                  # 49 taps with padding: compare-based bounds mode
    P(2, 16, 24, 24, 8, 6, 6, 1, 1, 2, 2),                  # 36 taps at stride 1: backward-data bitmask does not apply
    # backward-data row space: phases no tap reaches are dropped and dx zero-filled; taps spaced
    # dilation/stride apart when the stride divides the dilation
    P(4, 24, 15, 14, 40, 1, 1, 2, 2),                       # 1x1 stride 2: one phase of four
    P(3, 8, 17, 17, 12, 1, 1, 3, 3, 1, 2),                  # 1x1 stride 3 with padding: one phase of nine
    P(2, 6, 23, 21, 10, 2, 2, 4, 4, 0, 1),                  # 2x2 stride 4: phases {0, 1} of four (table)
    P(1, 16, 9, 9, 300, 1, 1, 2, 2),                        # zero fill together with a split reduction
    P(2, 12, 29, 29, 16, 5, 5, 1, 1, 4, 4, 2, 2),           # 5x5 dilation 2 stride 1: five spaced slots, not nine
    P(2, 8, 31, 30, 8, 3, 3, 2, 2, 2, 2, 4, 4),             # stride 2 dilation 4: one phase, slots two rows apart
    P(2, 8, 26, 26, 8, 3, 2, 3, 2, 1, 1, 2, 3, 2),          # neither divides: dense slots, all phases
    P(3, 12, 12, 14, 18, 3, 3, 2, 2, 1, 1, 2, 2, 3),        # three groups of 4 -> 6 channels on the GEMM tiles
]

# Thin groups: the direct kernels (one thread per output element; lanes = (position, tap) for the
# filter gradient).  Depthwise and channel multipliers, every parameter, tap counts that do and do
# not divide 64, more positions than one chunk, fewer images than splits.
DIRECT_CASES = [
    P(5, 24, 19, 17, 24, 3, 3, 1, 1, 1, 1, 1, 1, 24),          # depthwise 3x3
    P(3, 16, 22, 25, 32, 3, 3, 2, 2, 1, 1, 1, 1, 16),          # channel multiplier 2, stride 2
    P(2, 12, 15, 15, 12, 5, 5, 1, 1, 2, 2, 1, 1, 12),          # depthwise 5x5
    P(4, 10, 18, 21, 10, 3, 2, 2, 3, 1, 0, 2, 3, 10, 0),       # stride + dilation + no bias, non-square
    P(2, 8, 9, 9, 8, 1, 1, 1, 1, 0, 0, 1, 1, 8),               # depthwise 1x1 (a per-channel scale)
    P(3, 6, 31, 29, 6, 7, 7, 2, 2, 3, 3, 1, 1, 6),             # depthwise 7x7: one position per wave iteration
    P(1, 300, 6, 6, 300, 3, 3, 1, 1, 1, 1, 1, 1, 300),         # more pairs than a thousand / few images
    P(70, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 1, 4),              # many images per split
    P(2, 8, 12, 12, 8, 2, 2, 2, 2, 3, 3, 1, 1, 4),             # two channels per group, pad > kernel
    P(3, 10, 21, 18, 10, 3, 3, 1, 1, 2, 2, 2, 2, 10),          # 3x3 dilation 2 at stride 1
    P(2, 6, 14, 13, 6, 3, 3, 1, 1, 0, 0, 1, 1, 6),             # 3x3 without padding
    P(2, 6, 10, 11, 6, 3, 3, 1, 1, 4, 3, 1, 1, 6),             # pad beyond the kernel (mirrored pad negative)
    P(2, 14, 27, 26, 28, 5, 5, 2, 2, 2, 2, 1, 1, 14),          # 5x5 stride 2, channel multiplier 2
    P(2, 8, 13, 13, 8, 5, 5, 1, 1, 1, 3, 1, 2, 4),             # 5x5, two channels per group, mixed dilation
    P(3, 9, 23, 20, 9, 3, 3, 2, 2, 0, 0, 1, 1, 9),             # 3x3 stride 2 without padding (last row unread)
    P(2, 6, 16, 19, 12, 3, 3, 2, 2, 3, 2, 1, 1, 3),            # 3x3 stride 2, pad beyond the kernel, 2 -> 4 channels
    P(2, 5, 18, 17, 5, 5, 5, 2, 2, 1, 4, 1, 1, 5),             # 5x5 stride 2, uneven padding
    # "same" padding along rows of a multiple of four elements: four columns per thread, 16-byte accesses
    P(3, 7, 18, 12, 7, 3, 3, 1, 1, 1, 1, 1, 1, 7),             # 3x3, OH not a multiple of four
    P(2, 6, 9, 8, 12, 5, 5, 1, 1, 2, 2, 1, 1, 3),              # 5x5, two channels in and four out per group
    P(2, 5, 11, 20, 5, 3, 3, 1, 1, 0, 1, 1, 1, 5),             # no padding along the height
    P(2, 4, 7, 4, 4, 5, 5, 1, 1, 3, 2, 1, 1, 4),               # a single four-column block per row
    # the same at stride 2: two output columns per thread
    P(2, 6, 18, 16, 6, 3, 3, 2, 2, 1, 1, 1, 1, 6),             # 3x3 stride 2
    P(2, 4, 13, 12, 8, 5, 5, 2, 2, 2, 2, 1, 1, 4),             # 5x5 stride 2, channel multiplier 2, odd height
    P(3, 4, 10, 8, 4, 3, 3, 2, 2, 0, 1, 1, 1, 4),              # no padding along the height
    P(2, 4, 9, 20, 4, 3, 3, 2, 2, 3, 1, 1, 1, 2),              # two channels per group, tall padding
    P(1, 3, 3, 3, 3, 3, 3, 2, 2, 40, 37, 1, 1, 3),             # padding far larger than the image
    P(2, 16, 9, 10, 2, 3, 3, 2, 2, 1, 0, 1, 1, 2),             # eight channels in, one out per group
]

# Shapes that select the patch-staged kernel (256-column tiles of at most 48 rows; 128x128 and 32x128
# tiles for kernels of 25 taps or more): 8-aligned reduction channels, enough columns for the tile to win
# and for the grid not to want a split reduction.  (parameters, pass, the variant that pass must select)
PATCH_CASES = [
    (P(20, 48, 60, 45, 16, 5, 5, 1, 1, 2, 2), "bwd_data", "corr_m16_48x256x16_patch[es]"),  # 5x5, one image per many tiles
    (P(400, 96, 9, 9, 16, 3, 3, 1, 1, 1, 1, 1, 1, 2), "bwd_data", "corr_m16_48x256x16_patch[es]"),  # grouped, tiles span 4 images
    (P(49, 8, 32, 32, 8, 3, 3, 1, 1, 1, 1), "bwd_data", "corr_m16_16x256x16_patch[es]"),    # 16-row tile
    (P(12, 16, 70, 61, 48, 3, 5, 1, 1, 0, 3), "fwd", "corr_m16_48x256x16_patch[es]"),       # forward with 48 rows, ragged pad
    (P(33, 8, 32, 33, 20, 3, 3, 1, 1, 1, 1), "fwd", "corr_m32_32x256x16_patch[es]"),        # 32-row MFMA tile, forward
    (P(64, 8, 47, 49, 8, 3, 3, 2, 2, 1, 1), "bwd_data", "corr_m32_32x256x16_patch[er]"),    # 32-row tile, four sub-pixel phases
    (P(90, 8, 24, 25, 5, 3, 3, 1, 1, 1, 1), "fwd", "corr_m16_16x256x16_patch[es]"),         # 16-row tile, forward
    (P(100, 1, 48, 47, 8, 3, 3, 2, 2, 1, 1), "bwd_data", "corr_m16_16x256x16_patch[er]"),   # 16-row tile, sub-pixel scatter
    (P(64, 12, 48, 49, 8, 3, 3, 2, 2, 1, 1), "bwd_data", "corr_m16_48x256x16_patch[er]"),   # 48 rows = 12 channels x 4 phases
    (P(33, 20, 32, 33, 8, 3, 3, 1, 1, 1, 1), "bwd_data", "corr_m32_32x256x16_patch[es]"),   # 32-row tile at stride 1
    # kernels of 25 taps or more also take it on the 128x128 and 32x128 tiles (grids of more than 160 tiles)
    (P(24, 8, 30, 30, 128, 5, 5, 1, 1, 2, 2), "fwd", "corr_m32_128x128x16_patch[es]"),
    (P(24, 128, 30, 30, 8, 5, 5, 1, 1, 2, 2), "bwd_data", "corr_m32_128x128x16_patch[es]"),
    (P(48, 32, 41, 41, 8, 9, 9, 2, 2, 4, 4), "bwd_data", "corr_m32_128x128x16_patch[er]"),  # 9x9 at stride 2: 5x5 slots
    (P(100, 8, 16, 16, 32, 5, 5, 1, 1, 2, 2), "fwd", "corr_m32_32x128x16_patch[es]"),
    (P(100, 32, 16, 16, 8, 5, 5, 1, 1, 2, 2), "bwd_data", "corr_m32_32x128x16_patch[es]"),
    (P(48, 8, 41, 41, 8, 9, 9, 2, 2, 4, 4), "bwd_data", "corr_m32_32x128x16_patch[er]"),
]

# One cheap shape per (pass, tile, bounds mode) of the gather kernel and per (tile, bounds mode) of the
# filter-gradient kernel that none of the lists above selects.  Bounds modes: 0 = no padding, 1 = more
# than 32 taps (6x6, 7x7 kernels), 2 = at most 32 taps with padding (every backward-data pass has
# padding).  (parameters, pass, prefix of the variant that pass must select)
VARIANT_CASES = [
    (P(8, 1, 48, 49, 128, 1, 1), "fwd", "corr_m32_128x128x16[m0"),
    (P(8, 1, 47, 49, 128, 6, 6, 1, 1, 2, 2), "fwd", "corr_m32_128x128x16[m1"),
    (P(33, 128, 24, 25, 1, 6, 6), "bwd_data", "corr_m32_128x128x16[m1"),
    (P(8, 128, 48, 49, 1, 2, 2, 2, 2), "bwd_data", "corr_m32_128x128x16[m2"),
    (P(1, 1, 5, 6, 128, 2, 2, 2, 2), "fwd", "corr_m32_128x64x16[m0"),
    (P(1, 1, 5, 6, 128, 6, 6, 2, 2, 3, 3), "fwd", "corr_m32_128x64x16[m1"),
    (P(1, 128, 5, 6, 1, 6, 6, 1, 1, 2, 2), "bwd_data", "corr_m32_128x64x16[m1"),
    (P(1, 1, 5, 6, 96, 6, 6, 2, 2, 3, 3), "fwd", "corr_m32_96x128x16[m1"),
    (P(1, 1, 5, 6, 96, 3, 3, 2, 2, 1, 1), "fwd", "corr_m32_96x128x16[m2"),
    (P(1, 96, 5, 6, 1, 6, 6, 1, 1, 2, 2), "bwd_data", "corr_m32_96x128x16[m1"),
    (P(1, 96, 5, 6, 1, 1, 1), "bwd_data", "corr_m32_96x128x16[m2"),
    (P(8, 4, 48, 48, 64, 1, 1), "fwd", "corr_m32_64x128x16[m0"),
    (P(8, 1, 48, 49, 64, 6, 6, 1, 1, 2, 2), "fwd", "corr_m32_64x128x16[m1"),
    (P(8, 1, 48, 49, 64, 3, 3, 1, 1, 1, 1), "fwd", "corr_m32_64x128x16[m2"),
    (P(33, 64, 24, 25, 1, 6, 6), "bwd_data", "corr_m32_64x128x16[m1"),
    (P(8, 64, 48, 48, 4, 3, 3, 1, 1, 1, 1), "bwd_data", "corr_m32_64x128x16[m2"),
    (P(1, 1, 5, 6, 64, 6, 6, 2, 2, 3, 3), "fwd", "corr_m32_64x64x16[m1"),
    (P(1, 64, 5, 6, 1, 6, 6, 1, 1, 2, 2), "bwd_data", "corr_m32_64x64x16[m1"),
    (P(64, 1, 24, 25, 20, 6, 6, 1, 1, 2, 2), "fwd", "corr_m32_32x256x16[m1"),
    (P(64, 20, 24, 25, 1, 6, 6), "bwd_data", "corr_m32_32x256x16[m1"),
    (P(33, 40, 48, 49, 1, 2, 2, 2, 2), "bwd_data", "corr_m32_32x256x16[m2"),
    (P(4, 20, 12, 13, 1, 6, 6), "bwd_data", "corr_m32_32x128x16[m1"),
    (P(8, 1, 48, 49, 130, 1, 1), "fwd", "corr_m16_48x256x16[m0"),
    (P(8, 1, 48, 49, 130, 6, 6, 1, 1, 2, 2), "fwd", "corr_m16_48x256x16[m1"),
    (P(8, 1, 48, 49, 130, 3, 3, 1, 1, 1, 1), "fwd", "corr_m16_48x256x16[m2"),
    (P(33, 130, 24, 25, 1, 6, 6), "bwd_data", "corr_m16_48x256x16[m1"),
    (P(8, 130, 48, 49, 1, 2, 2, 2, 2), "bwd_data", "corr_m16_48x256x16[m2"),
    (P(1, 1, 5, 6, 33, 6, 6, 2, 2, 3, 3), "fwd", "corr_m16_48x128x16[m1"),
    (P(1, 40, 5, 6, 1, 6, 6, 1, 1, 2, 2), "bwd_data", "corr_m16_48x128x16[m1"),
    (P(2, 1, 48, 49, 200, 1, 1), "fwd", "corr_m16_16x256x16[m0"),
    (P(8, 1, 24, 25, 200, 6, 6, 1, 1, 2, 2), "fwd", "corr_m16_16x256x16[m1"),
    (P(33, 1, 9, 10, 200, 3, 3, 1, 1, 2, 2), "fwd", "corr_m16_16x256x16[m2"),
    (P(33, 6, 40, 41, 1, 6, 6, 1, 1, 0, 0, 2, 2), "bwd_data", "corr_m16_16x256x16[m1"),
    (P(8, 4, 48, 49, 128, 3, 3, 1, 1, 1, 1), "fwd", "corr_m32_128x128x16[m2"),
    (P(64, 1, 28, 28, 20, 5, 5), "fwd", "corr_m32_32x256x16[m0"),
    (P(100, 3, 32, 32, 32, 5, 5, 1, 1, 2, 2), "fwd", "corr_m32_32x256x16[m2"),
    (P(1, 18, 28, 35, 54, 6, 7, 3, 4, 5, 1, 2, 2, 2), "fwd", "corr_m32_32x128x16[m1"),
    (P(90, 8, 24, 25, 5, 3, 3, 1, 1, 1, 1), "bwd_data", "corr_m16_16x256x16[m2"),
    (P(2, 3, 7, 6, 60, 3, 3, 2, 2, 1, 1), "fwd", "corr_m32_64x64x16[m2"),
    (P(1, 8, 5, 6, 128, 3, 3), "bwd_filter", "wgrad_m32_128x128x32[m0"),
    (P(1, 3, 5, 6, 128, 6, 6, 2, 2, 3, 3), "bwd_filter", "wgrad_m32_128x128x32[m1"),
    (P(1, 3, 5, 6, 96, 6, 6, 2, 2, 3, 3), "bwd_filter", "wgrad_m32_96x128x32[m1"),
    (P(1, 1, 5, 6, 96, 6, 6, 2, 2, 3, 3), "bwd_filter", "wgrad_m32_128x64x32[m1"),
    (P(1, 1, 5, 6, 96, 3, 3, 2, 2, 1, 1), "bwd_filter", "wgrad_m32_128x64x32[m2"),
    # the 64-row filter-gradient tile is kept for grids of 256 workgroups or more (48 outputs, 4 column tiles, 86 splits)
    (P(6, 48, 66, 66, 48, 3, 3), "bwd_filter", "wgrad_m32_64x128x32[m0"),
    (P(6, 48, 64, 64, 48, 3, 3, 1, 1, 2, 2, 2, 2), "bwd_filter", "wgrad_m32_64x128x32[m1"),
    # at most four GEMM rows per group: corr_thin_kernel, rows x bounds modes (several 64-column workgroups each)
    (P(8, 1, 13, 14, 2, 1, 1, 2, 2), "fwd", "corr_thin_r2[m0"),
    (P(3, 1, 24, 25, 2, 6, 6, 2, 2, 1, 1, 2, 2), "fwd", "corr_thin_r2[m1"),
    (P(8, 1, 13, 14, 3, 1, 1, 2, 2), "fwd", "corr_thin_r3[m0"),
    (P(3, 1, 24, 25, 4, 6, 6, 2, 2, 1, 1, 2, 2), "fwd", "corr_thin_r4[m1"),
    (P(3, 2, 13, 14, 1, 6, 6, 1, 1, 0, 0, 2, 2), "bwd_data", "corr_thin_r2[m1"),
    (P(3, 3, 13, 14, 1, 6, 6, 1, 1, 0, 0, 2, 2), "bwd_data", "corr_thin_r3[m1"),
    (P(3, 4, 13, 14, 1, 6, 6, 1, 1, 0, 0, 2, 2), "bwd_data", "corr_thin_r4[m1"),
    (P(5, 4, 21, 19, 7, 4, 4, 1, 1, 1, 1), "bwd_data", "corr_thin_r4[m2"),
    (P(8, 1, 13, 14, 4, 1, 1, 2, 2), "fwd", "corr_thin_r4[m0"),
    # the same with the gathered rows staged in LDS (stride 1, dilation 1, 3x3 or 5x5 taps): rows x tap width, both
    # passes; tiles of 128 columns that span several images, ragged last tile, asymmetric and over-sized padding,
    # channel counts that are no multiple of the four waves, groups
    (P(4, 20, 17, 23, 1, 3, 3, 1, 1, 1, 1), "fwd", "corr_thin_r1_lds3"),
    (P(6, 7, 16, 15, 2, 3, 3, 1, 1, 0, 1), "fwd", "corr_thin_r2_lds3"),
    (P(6, 6, 16, 15, 3, 3, 3, 1, 1, 2, 2), "fwd", "corr_thin_r3_lds3"),
    (P(5, 9, 21, 19, 4, 3, 3), "fwd", "corr_thin_r4_lds3"),
    (P(3, 5, 30, 29, 1, 5, 5, 1, 1, 1, 2), "fwd", "corr_thin_r1_lds5"),
    (P(7, 3, 12, 11, 2, 5, 5, 1, 1, 2, 2), "fwd", "corr_thin_r2_lds5"),
    (P(7, 3, 12, 11, 3, 5, 5, 1, 1, 2, 2), "fwd", "corr_thin_r3_lds5"),
    (P(6, 8, 15, 16, 8, 5, 5, 1, 1, 2, 2, 1, 1, 2), "fwd", "corr_thin_r4_lds5"),
    (P(9, 1, 10, 9, 17, 3, 3), "bwd_data", "corr_thin_r1_lds3"),
    (P(4, 2, 25, 27, 5, 3, 3, 1, 1, 0, 2), "bwd_data", "corr_thin_r2_lds3"),
    (P(4, 3, 25, 27, 5, 3, 3, 1, 1, 1, 1), "bwd_data", "corr_thin_r3_lds3"),
    (P(5, 4, 21, 19, 7, 3, 3, 1, 1, 1, 1), "bwd_data", "corr_thin_r4_lds3"),
    (P(3, 1, 33, 31, 6, 5, 5, 1, 1, 2, 2), "bwd_data", "corr_thin_r1_lds5"),
    (P(7, 2, 12, 11, 6, 5, 5, 1, 1, 2, 2), "bwd_data", "corr_thin_r2_lds5"),
    (P(3, 3, 20, 31, 9, 5, 5, 1, 1, 4, 4), "bwd_data", "corr_thin_r3_lds5"),
    (P(6, 8, 15, 16, 8, 5, 5, 1, 1, 2, 2, 1, 1, 2), "bwd_data", "corr_thin_r4_lds5"),
]


def _valid(pd):
    return (oracle.out_size(pd["h"], pd["kernel_h"], pd["stride_h"], pd["pad_h"], pd["dilation_h"]) >= 1 and
            oracle.out_size(pd["w"], pd["kernel_w"], pd["stride_w"], pd["pad_w"], pd["dilation_w"]) >= 1)


def random_params(rng):
    """One random, valid parameter set with a small oracle cost."""
    while True:
        g = int(rng.choice([1, 1, 1, 2, 3, 4]))
        c = g * int(rng.integers(1, 9))
        k = g * int(rng.integers(1, 13))
        kh, kw = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        sh, sw = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        dh, dw = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        ph, pw = int(rng.integers(0, 5)), int(rng.integers(0, 5))
        h, w = int(rng.integers(1, 24)), int(rng.integers(1, 24))
        n = int(rng.integers(1, 6))
        pd = dict(n=n, c=c, h=h, w=w, num_output=k, kernel_h=kh, kernel_w=kw, stride_h=sh, stride_w=sw, pad_h=ph,
                  pad_w=pw, dilation_h=dh, dilation_w=dw, group=g, bias_term=int(rng.integers(0, 2)))
        if _valid(pd):
            return pd


def random_thin_group_params(rng):
    """Random depthwise-like parameter sets: many groups of one or two channels, 3x3 and 5x5 kernels
    (the rows-per-thread kernels) and arbitrary ones (the general direct kernels)."""
    while True:
        g = int(rng.integers(2, 13))
        c, k = g * int(rng.integers(1, 3)), g * int(rng.integers(1, 4))
        kh, kw = [(3, 3), (5, 5), (int(rng.integers(1, 8)), int(rng.integers(1, 8)))][int(rng.integers(0, 3))]
        sh, sw = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        if rng.integers(0, 2):
            sh = sw = 1
        dh, dw = int(rng.integers(1, 3)), int(rng.integers(1, 3))
        ph, pw = int(rng.integers(0, 5)), int(rng.integers(0, 5))
        h, w = int(rng.integers(1, 30)), int(rng.integers(1, 30))
        pd = dict(n=int(rng.integers(1, 7)), c=c, h=h, w=w, num_output=k, kernel_h=kh, kernel_w=kw, stride_h=sh,
                  stride_w=sw, pad_h=ph, pad_w=pw, dilation_h=dh, dilation_w=dw, group=g,
                  bias_term=int(rng.integers(0, 2)))
        if _valid(pd):
            return pd


def random_multi_tile_params(rng):
    """Random parameter sets large enough for several tiles per dimension (up to 4e8 FLOPs per pass)."""
    while True:
        g = int(rng.choice([1, 1, 2, 4, 8]))
        c, k = g * int(rng.integers(1, 12)), g * int(rng.integers(1, 40))
        kh, kw = int(rng.integers(1, 8)), int(rng.integers(1, 8))
        sh, sw = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        dh, dw = int(rng.integers(1, 3)), int(rng.integers(1, 3))
        ph, pw = int(rng.integers(0, 7)), int(rng.integers(0, 7))
        h, w = int(rng.integers(1, 50)), int(rng.integers(1, 50))
        n = int(rng.integers(1, 9))
        pd = dict(n=n, c=c, h=h, w=w, num_output=k, kernel_h=kh, kernel_w=kw, stride_h=sh, stride_w=sw, pad_h=ph,
                  pad_w=pw, dilation_h=dh, dilation_w=dw, group=g, bias_term=int(rng.integers(0, 2)))
        if not _valid(pd):
            continue
        oh = oracle.out_size(h, kh, sh, ph, dh)
        ow = oracle.out_size(w, kw, sw, pw, dw)
        if 2.0 * n * k * (c // g) * kh * kw * oh * ow < 4e8:
            return pd


def random_many_channel_params(rng):
    """Random layers with about 128 or 256 output channels per group and a reduced dimension of
    100-500: the 128x128 backward-filter tile with ragged rows and columns, every bounds mode."""
    while True:
        g = int(rng.choice([1, 1, 2]))
        # rows and reduced dimension a little below a multiple of 128: the tile that pads least
        k = g * (128 * int(rng.integers(1, 3)) - int(rng.integers(0, 20)))
        kh, kw = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        c = g * max(1, (128 * int(rng.integers(1, 5)) - int(rng.integers(0, 12))) // (kh * kw))
        sh, sw = int(rng.integers(1, 3)), int(rng.integers(1, 3))
        ph, pw = int(rng.integers(0, 3)), int(rng.integers(0, 3))
        dh = dw = int(rng.choice([1, 1, 2]))
        h, w = int(rng.integers(4, 16)), int(rng.integers(4, 16))
        pd = dict(n=int(rng.integers(1, 5)), c=c, h=h, w=w, num_output=k, kernel_h=kh, kernel_w=kw, stride_h=sh,
                  stride_w=sw, pad_h=ph, pad_w=pw, dilation_h=dh, dilation_w=dw, group=g,
                  bias_term=int(rng.integers(0, 2)))
        if _valid(pd):
            return pd


def random_thin_row_params(rng):
    """Random layers with at most four input channels or at most four outputs per group at stride 1, mostly 3x3 and
    5x5 kernels: GEMMs of at most four rows (the thin-row kernel and its LDS-staged form), with images small enough
    that a 128-column tile spans several of them and large enough that it does not, padding up to past the kernel."""
    while True:
        g = int(rng.choice([1, 1, 1, 2, 3]))
        few, many = int(rng.integers(1, 5)), int(rng.integers(1, 24))
        c, k = (g * few, g * many) if rng.integers(0, 2) else (g * many, g * few)
        kh, kw = [(3, 3), (5, 5), (3, 3), (5, 5), (int(rng.integers(1, 7)), int(rng.integers(1, 7)))][int(rng.integers(0, 5))]
        ph, pw = int(rng.integers(0, kh + 1)), int(rng.integers(0, kw + 1))
        h, w = int(rng.integers(1, 45)), int(rng.integers(1, 45))
        pd = dict(n=int(rng.integers(1, 9)), c=c, h=h, w=w, num_output=k, kernel_h=kh, kernel_w=kw, stride_h=1,
                  stride_w=1, pad_h=ph, pad_w=pw, dilation_h=1, dilation_w=1, group=g,
                  bias_term=int(rng.integers(0, 2)))
        if _valid(pd):
            return pd


# Seeds and counts of the seeded random tests (test_random_sweep_gpu.py draws exactly these).
RANDOM_BLOCKS = [(20260 + b, 12, random_params) for b in range(6)]
THIN_BLOCKS = [(50500 + b, 12, random_thin_group_params) for b in range(4)]
THIN_ROW = (80800, 48, random_thin_row_params)
MULTI_TILE = (60600, 40, random_multi_tile_params)
MANY_CHANNEL = (70700, 16, random_many_channel_params)


def draw_block(seed, count, gen):
    rng = np.random.default_rng(seed)
    return [gen(rng) for _ in range(count)]


# InnerProduct shapes (m, k, num_output): ragged against every tile size, tiny, tall, wide
IP_SHAPES = [
    (1, 1, 1), (1, 4, 1), (3, 7, 5), (5, 33, 129), (64, 500, 10), (64, 800, 500), (37, 1000, 130), (130, 257, 70),
    (128, 2048, 96), (16, 4100, 48), (200, 64, 1000), (9, 16, 2050),
]
# beta = 1 (the filter gradient is added to what dw holds).  The last three: at most four outputs -- the sum then
# happens in the epilogue of the kernel for GEMMs of at most four rows -- and at most four batch rows (that kernel
# computes dx).
IP_BETA_SHAPES = [(64, 800, 500), (130, 257, 70), (9, 16, 2050), (37, 300, 3), (20, 1000, 1), (3, 129, 40)]
IP_RANDOM = (777, 16)


def random_ip_case(rng):
    m, k, o = int(rng.integers(1, 200)), int(rng.integers(1, 700)), int(rng.integers(1, 300))
    relu, bias = int(rng.integers(0, 2)), bool(rng.integers(0, 2))
    return m, k, o, relu, bias


def fp32_conv_cases():
    """Every convolution parameter set the default `-m gpu` run sends through the fp32 entry points."""
    from paper_1810_02272_amd import workloads

    out = list(SWEEP) + list(DIRECT_CASES) + [c[0] for c in PATCH_CASES] + [c[0] for c in VARIANT_CASES]
    out += [l.params_dict() for l in workloads.LAYERS + workloads.DW_LAYERS]
    for blk in RANDOM_BLOCKS + THIN_BLOCKS + [THIN_ROW, MULTI_TILE, MANY_CHANNEL]:
        out += draw_block(*blk)
    return out


def fp64_conv_cases():
    """The same for the double entry points."""
    from paper_1810_02272_amd import workloads

    out = list(SWEEP) + list(DIRECT_CASES) + [c[0] for c in VARIANT_CASES]
    out += [l.params_dict() for l in workloads.LAYERS]
    for blk in RANDOM_BLOCKS + THIN_BLOCKS + [THIN_ROW, MULTI_TILE, MANY_CHANNEL]:
        out += draw_block(*blk)
    return out
