"""Small convolution shapes that exercise the edges of the tiling (shared by host and GPU tests)."""
from paper_2002_02145_amd.workloads import ConvShape

EDGE_SHAPES = [
    ConvShape(1, 64, 14, 14, 64, 3, 3, 1, 1, "cfg1"),
    ConvShape(3, 32, 7, 7, 64, 3, 3, 1, 1, "tiles_cross_images"),      # 49 px per image: tiles span images
    ConvShape(2, 3, 23, 19, 32, 7, 7, 2, 3, "stem_like_C3"),            # ragged C, big filter, stride 2
    ConvShape(2, 48, 9, 11, 32, 1, 1, 2, 0, "1x1_stride2_odd"),
    ConvShape(1, 20, 6, 5, 16, 2, 3, 1, 1, "non_square_filter"),        # K = 16: half an MFMA tile
    ConvShape(5, 16, 5, 5, 128, 1, 1, 1, 0, "1x1_small"),
    ConvShape(1, 16, 1, 1, 16, 1, 1, 1, 0, "single_pixel"),
    ConvShape(2, 16, 4, 4, 32, 3, 3, 3, 2, "stride3_pad2"),
    ConvShape(1, 32, 12, 12, 256, 3, 3, 1, 0, "no_pad_K256"),
    ConvShape(2, 16, 6, 6, 48, 3, 3, 1, 1, "K48_ragged_tile"),
    ConvShape(1, 80, 3, 3, 96, 1, 1, 1, 0, "five_blocks_prime_batch"),  # batch-reduce length 5
    ConvShape(2, 4, 9, 10, 16, 7, 7, 1, 3, "7x7_C4_stride1"),           # tap-packed path with all 4 lanes real
    ConvShape(1, 5, 9, 9, 32, 7, 7, 2, 3, "7x7_C5_not_packed"),         # one channel too many for tap packing
    ConvShape(3, 64, 9, 7, 256, 1, 1, 1, 0, "1x1_64to256_tiles_cross_images"),  # pixel-stationary kernels, ragged tail
    ConvShape(2, 50, 10, 10, 512, 1, 1, 2, 0, "1x1_C50_K512_stride2"),  # the same with zero lanes, two channel groups
    ConvShape(2, 3, 20, 17, 64, 7, 7, 2, 3, "stem_like_K64"),           # tap-packed 7x7 in the 16x16-tile kernels too
    ConvShape(1, 64, 5, 5, 240, 1, 1, 1, 1, "1x1_64to240_pad1"),        # ... last channel block missing, padded border
    ConvShape(2, 3, 18, 15, 128, 7, 7, 2, 3, "stem_like_K128"),         # tap-packed 7x7 on the wide channel tiles
    ConvShape(1, 7, 11, 12, 96, 7, 7, 1, 3, "7x7_C7_K96"),              # 16-bit packing uses 8 channel lanes; K = 96 pads a 64-wide tile
    # tap-packed loops of the other filter sides (first layers of image networks)
    ConvShape(2, 3, 13, 11, 32, 3, 3, 2, 1, "3x3s2_C3_K32"),            # 9 taps: 3 (fp32) / 5 (16-bit) batch elements
    ConvShape(2, 3, 9, 12, 64, 3, 3, 1, 1, "3x3s1p1_C3_K64"),           # 16-bit: the patch loop has first call here
    ConvShape(1, 2, 12, 10, 48, 5, 5, 1, 2, "5x5_C2_K48"),
    ConvShape(2, 3, 35, 31, 64, 11, 11, 4, 2, "11x11s4_C3_K64"),        # 121 taps: 31 / 61 batch elements
    ConvShape(1, 3, 27, 23, 96, 11, 11, 4, 0, "11x11s4_C3_K96_nopad"),
    ConvShape(1, 6, 10, 9, 32, 5, 5, 2, 2, "5x5_C6_K32"),               # packed in 16 bits only
    ConvShape(1, 4, 8, 8, 16, 3, 3, 1, 1, "3x3_C4_fp32_not_packed"),    # four channels: only 7x7 packs them in fp32
    # loops with a 5x5 filter baked in
    ConvShape(2, 32, 9, 11, 64, 5, 5, 1, 2, "5x5_C32_K64"),
    ConvShape(1, 48, 13, 8, 96, 5, 5, 2, 1, "5x5s2_C48_K96"),           # three c-blocks: rings of 2 and 4 both pad the range
]
