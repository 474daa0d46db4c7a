"""Shapes that reach every instantiation of the product kernel.

Key: (workgroup tile rows, tile columns, paired scale fetch (K a multiple of 256), K split); value: (M, N, K) for which
the planner picks exactly that variant.  All are ragged (M not a multiple of 64, N not a multiple of 4).  A test without
a GPU checks the planner's choice for each, so the GPU parity test over this table is known to run all of them.
"""

VARIANT_SHAPES = {
    (128, 128, False, False): (77, 6, 64),
    (128, 128, False, True): (71, 6, 1152),
    (128, 128, True, False): (16751, 578, 256),
    (128, 128, True, True): (12226, 17, 4096),
    (128, 192, True, False): (12, 5, 256),
    (128, 192, True, True): (13, 7, 1024),
    (128, 256, False, False): (2593, 2955, 64),
    (128, 256, False, True): (10762, 150, 1856),
    (128, 256, True, False): (2860, 2774, 256),
    (128, 256, True, True): (3105, 393, 2560),
    (256, 128, False, False): (18382, 131, 64),
    (256, 128, False, True): (16416, 5, 1216),
    (256, 128, True, False): (16951, 201, 256),
    (256, 128, True, True): (4857, 7, 3584),
    (256, 256, False, False): (19641, 521, 64),
    (256, 256, False, True): (11069, 134, 2880),
    (256, 256, True, False): (14086, 783, 256),
    (256, 256, True, True): (16564, 193, 3072),
}

# The same for operands with 1 x 128 outer blocks (K a multiple of 128; no 256 x 256 tile there: that mode keeps two
# accumulator sets per wave).
VARIANT_SHAPES_BLOCK128 = {
    (128, 128, False, False): (13242, 73, 128),
    (128, 128, False, True): (731, 137, 1152),
    (128, 128, True, False): (16897, 2141, 512),
    (128, 128, True, True): (13657, 41, 3584),
    (128, 192, True, False): (181, 1495, 256),
    (128, 192, True, True): (126, 2773, 2048),
    (128, 256, False, False): (6452, 2450, 1408),
    (128, 256, False, True): (6439, 171, 2944),
    (128, 256, True, False): (2628, 2958, 512),
    (128, 256, True, True): (10813, 206, 3072),
    (256, 128, False, False): (18350, 263, 1408),
    (256, 128, False, True): (4409, 281, 1920),
    (256, 128, True, False): (6332, 2378, 512),
    (256, 128, True, True): (3661, 225, 3584),
}
