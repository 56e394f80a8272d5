"""Pins of the requirement-derivation checker (oracle/probes.cpp) that do not come from the library.

Sec. III-A of the paper: a task's requirements are the sum of its device allocations and the
geometry of its launches.  Footprints below are worked out by hand from the buffer lists; grids
are held to "whole tiles of one of the kernel's tile shapes cover the output"; workgroups per CU
follow from the CU's budgets (160 KiB of LDS, 4 SIMDs x 512 vector registers per lane, 32 wave
slots) and each kernel's own use of them.  The library's probes are compared with the checker in
test_abi_host.py; here the checker itself is held to figures fixed outside both."""
import ctypes as C
import itertools

import pytest

import oracle

U = C.c_uint64
KIB = 1024


def _lib():
    lib = oracle.lib()
    for f in ("orc_jacobi_residency", "orc_gemm_f32_residency", "orc_gemm_bf16_residency", "orc_conv3x3_residency",
              "orc_bfs_residency"):
        getattr(lib, f).restype = C.c_uint64
    return lib


def _probe(fn, *args):
    out = (U * 7)()
    getattr(_lib(), fn)(*[U(a) for a in args], out)
    return list(out)


def _cnn_probe(layers, batch, h, w):
    flat = (U * (3 * len(layers)))(*[x for L in layers for x in L])
    out = (U * 7)()
    _lib().orc_cnn_probe(flat, U(len(layers)), U(batch), U(h), U(w), out)
    return list(out)


def ceil_div(a, b):
    return -(-a // b)


def round8(x):
    return ceil_div(x, 8) * 8


# ------------------------------------------------------------------ footprints, by hand
def test_footprints_of_the_configured_tasks():
    # Jacobi 16384^2: two fp32 grids = 2 GiB; 4096^2: 128 MiB
    assert _probe("orc_jacobi_probe", 16384, 50)[0] == 2 << 30
    assert _probe("orc_jacobi_probe", 4096, 100)[0] == 128 << 20
    # fp32 GEMM 32768^3: three fp32 matrices = 12 GiB; 4096^3: 192 MiB; 256^3: 768 KiB
    assert _probe("orc_gemm_f32_probe", 32768, 32768, 32768)[0] == 12 << 30
    assert _probe("orc_gemm_f32_probe", 4096, 4096, 4096)[0] == 192 << 20
    assert _probe("orc_gemm_f32_probe", 256, 256, 256)[0] == 768 * KIB
    # bf16 GEMM 4096^3: two bf16 operands of 32 MiB + one fp32 result of 64 MiB
    assert _probe("orc_gemm_bf16_probe", 4096, 4096, 4096)[0] == 134217728
    # ... and two small ragged shapes: (m k + k n) * 2 + m n * 4
    assert _probe("orc_gemm_bf16_probe", 100, 72, 64)[0] == (6400 + 4608) * 2 + 7200 * 4 == 50816
    assert _probe("orc_gemm_bf16_probe", 3, 5, 7)[0] == (21 + 35) * 2 + 15 * 4 == 172
    # BFS 2^20 vertices, 2^24 stored edges: row pointers 4 MiB + 4, columns 64 MiB, levels 4 MiB,
    # two queues of 4 MiB, three bitmaps of 128 KiB, 256 bytes of counters
    assert _probe("orc_bfs_probe", 1 << 20, 1 << 24)[0] == 4194308 + 67108864 + 4194304 + 8388608 + 393216 + 256 == 84279556
    # 1000 vertices, 3000 edges: 4004 + 12000 + 4000; queues 4000 -> 4096 each; a bitmap is 32 words
    # -> 64 words = 256 bytes, three of them; 256 bytes of counters
    assert _probe("orc_bfs_probe", 1000, 3000)[0] == 4004 + 12000 + 4000 + 8192 + 768 + 256 == 29220
    # 1 vertex, no edge: 8 + 0 + 4; queues 4 -> 256 each; bitmaps 256 each; counters
    assert _probe("orc_bfs_probe", 1, 0)[0] == 8 + 4 + 512 + 768 + 256 == 1548


def test_footprints_of_conv_layers_and_of_the_ten_layer_net():
    # one layer: bf16 input + bf16 weights + bf16 output
    # batch 2, 8x8, 32 -> 64 channels, stride 2: output 4x4
    assert _probe("orc_conv3x3_probe", 2, 8, 8, 32, 64, 2)[0] == (2 * 64 * 32 + 9 * 32 * 64 + 2 * 16 * 64) * 2 == 49152
    # batch 1, 5x7, 3 -> 8 channels, stride 1: output 5x7
    assert _probe("orc_conv3x3_probe", 1, 5, 7, 3, 8, 1)[0] == (105 + 216 + 280) * 2 == 1202
    # odd size, stride 2: 13 -> 7
    assert _probe("orc_conv3x3_probe", 1, 13, 13, 8, 8, 2)[0] == (13 * 13 * 8 + 9 * 64 + 7 * 7 * 8) * 2 == 4640
    # the 10-layer net on 416 x 416 x 3 (channels 32, 64, 64, 128, 128, 256, 256, 512, 512, 512; every
    # second layer has stride 2): 7 060 320 weights = 14.1 MB; the largest intermediate activation is
    # layer 1's, 416 * 416 * 32 bf16 = 11.1 MB per image, held twice; input 416 * 416 * 3 bf16;
    # output 13 * 13 * 512 fp32
    net = [(3, 32, 1), (32, 64, 2), (64, 64, 1), (64, 128, 2), (128, 128, 1), (128, 256, 2), (256, 256, 1),
           (256, 512, 2), (512, 512, 1), (512, 512, 2)]
    params = 9 * (96 + 2048 + 4096 + 8192 + 16384 + 32768 + 65536 + 131072 + 262144 + 262144)
    assert params == 7060320
    for batch, want in ((1, 37656256), (8, 202405568)):
        by_hand = batch * 1038336 + 2 * params + 2 * batch * 11075584 + batch * 346112
        assert by_hand == want
        assert _cnn_probe(net, batch, 416, 416)[0] == want
    # a two-layer chain on a 6x6 image, batch 3: input 3*36*8 bf16, weights 9*(8*16 + 16*4) bf16, the only
    # intermediate is 3*36*16 bf16 (twice), output 3*9*4 fp32 (second layer stride 2: 6 -> 3)
    assert _cnn_probe([(8, 16, 1), (16, 4, 2)], 3, 6, 6)[0] == 1728 + 3456 + 2 * 3456 + 432 == 12528
    # a single layer as a chain: no intermediate at all
    assert _cnn_probe([(8, 16, 1)], 1, 4, 4)[0] == 4 * 4 * 8 * 2 + 9 * 8 * 16 * 2 + 4 * 4 * 16 * 4 == 3584


# ------------------------------------------------------------------ grids: whole tiles cover the output
F32_TILES = {(64, 256), (128, 512), (256, 256)}                       # (square tile side, threads)
BF16_TILES = {((256, 256), 256), ((128, 128), 256), ((128, 256), 256)}


@pytest.mark.parametrize("m,n,k", list(itertools.product((1, 63, 64, 200, 1000, 4096, 5000), (1, 8, 130, 1024, 4100), (1, 16, 48, 64)))
                         + [(4096, 4096, 4096), (32768, 32768, 32768), (8192, 8192, 16), (1024, 1024, 1024)])
def test_gemm_grids_are_whole_tiles_of_one_of_the_tile_shapes(m, n, k):
    out = _probe("orc_gemm_f32_probe", m, n, k)
    assert out[2:4] == [1, 1] and out[5:7] == [1, 1]
    fits = [(t, th) for t, th in F32_TILES if out[1] == round8(ceil_div(m, t) * ceil_div(n, t)) and out[4] == th]
    assert fits, (m, n, k, out)
    assert out[1] * max(t for t, _ in fits) ** 2 >= m * n                  # the grid covers C
    out = _probe("orc_gemm_bf16_probe", m, n, k)
    fits = [t for t, th in BF16_TILES if out[1] == round8(ceil_div(m, t[0]) * ceil_div(n, t[1])) and out[4] == th]
    assert fits, (m, n, k, out)
    assert out[1] * max(t[0] * t[1] for t in fits) >= m * n


def test_the_configured_gemms_get_the_tiles_that_fill_the_device():
    # 4096^3: 16 x 16 tiles of 256 x 256 = one per CU of the 256; 32768^3: 128 x 128 of them
    assert _probe("orc_gemm_f32_probe", 4096, 4096, 4096)[1:] == [256, 1, 1, 256, 1, 1]
    assert _probe("orc_gemm_f32_probe", 32768, 32768, 32768)[1] == 16384
    assert _probe("orc_gemm_bf16_probe", 4096, 4096, 4096)[1:] == [256, 1, 1, 256, 1, 1]
    # 256^3 (the smoke mix): too few big tiles, 4 x 4 tiles of 64 x 64
    assert _probe("orc_gemm_f32_probe", 256, 256, 256)[1:] == [16, 1, 1, 256, 1, 1]
    # 1024^3 in bf16: 16 big tiles would leave 240 CUs idle -> 8 x 8 tiles of 128 x 128
    assert _probe("orc_gemm_bf16_probe", 1024, 1024, 1024)[1] == 64


def test_fp32_gemm_tile_is_the_one_its_busiest_cu_finishes_first():
    # cost of a tile shape = tiles the busiest of the 256 CUs works off x tile area x (100000 // TFLOP/s of that tile)
    # 2176^3: 256 x 256: 81 tiles -> 1 x 65536 x 653 = 42.8 M; 128 x 128: 289 -> 2 x 16384 x 666 = 21.8 M;
    #         64 x 64: 1156 -> 5 x 4096 x 699 = 14.3 M: the small tile, 34 x 34 of them
    assert _probe("orc_gemm_f32_probe", 2176, 2176, 2176)[1:] == [1160, 1, 1, 256, 1, 1]
    # 2816^3: 128 x 128: 484 -> 2 x 16384 x 666 = 21.8 M; 64 x 64: 1936 -> 8 x 4096 x 699 = 22.9 M; 256 x 256: 121 -> 42.8 M
    assert _probe("orc_gemm_f32_probe", 2816, 2816, 2816)[1:] == [488, 1, 1, 512, 1, 1]
    # 4160^3: 256 x 256: 289 -> 2 x 65536 x 653 = 85.6 M; 128 x 128: 1089 -> 5 x 16384 x 666 = 54.6 M; 64 x 64: 4225 -> 17 x 4096 x 699 = 48.7 M
    assert _probe("orc_gemm_f32_probe", 4160, 4160, 4160)[1:] == [4232, 1, 1, 256, 1, 1]
    # 6848^3 (k > 5632: the small tile counts 100000 // 128 = 781): 256 x 256: 729 -> 3 x 65536 x 653 = 128.4 M;
    #         128 x 128: 2916 -> 12 x 16384 x 666 = 130.9 M; 64 x 64: 11449 -> 45 x 4096 x 781 = 144.0 M
    assert _probe("orc_gemm_f32_probe", 6848, 6848, 6848)[1:] == [736, 1, 1, 256, 1, 1]
    # 1792^3: 128 x 128: 196 -> 1 x 16384 x 666 = 10.9 M; 64 x 64: 784 -> 4 x 4096 x 699 = 11.5 M
    assert _probe("orc_gemm_f32_probe", 1792, 1792, 1792)[1:] == [200, 1, 1, 512, 1, 1]
    # a tall shape: 8192 x 512 x 1024: 256 x 256: 64 tiles -> 42.8 M; 128 x 128: 256 -> 10.9 M; 64 x 64: 1024 -> 4 x 4096 x 699 = 11.5 M
    assert _probe("orc_gemm_f32_probe", 8192, 512, 1024)[1:] == [256, 1, 1, 512, 1, 1]


CONV_TILES = [((128, 128), 256), ((256, 64), 256), ((64, 64), 256), ((64, 64), 64), ((128, 64), 256)]


@pytest.mark.parametrize("shape", [(1, 416, 416, 3, 32, 1), (8, 416, 416, 32, 64, 2), (2, 13, 11, 512, 512, 2), (1, 5, 6, 5, 7, 1),
                                   (3, 26, 26, 40, 200, 1), (8, 104, 104, 128, 128, 1), (1, 104, 104, 128, 128, 1),
                                   (8, 26, 26, 512, 512, 2), (2, 416, 416, 3, 64, 1), (1, 64, 64, 3, 36, 1), (4, 208, 208, 64, 64, 1),
                                   (1, 52, 52, 96, 72, 1), (7, 9, 9, 32, 8, 1), (1, 1, 1, 64, 64, 1)])
def test_conv_grids_cover_pixels_times_channels(shape):
    b, h, w, ci, co, st = shape
    out = _probe("orc_conv3x3_probe", *shape)
    pixels = b * ceil_div(h, st) * ceil_div(w, st)                     # pad 1, 3x3: out = ceil(in / stride)
    fits = [t for t, th in CONV_TILES if out[1] == round8(ceil_div(pixels, t[0]) * ceil_div(co, t[1])) and out[4] == th]
    if ci == 3 and co <= 64:                                           # first-layer kernel: 256 pixels, all channels
        fits += [(256, co)] if out[1] == round8(ceil_div(pixels, 256)) and out[4] == 256 else []
    if st == 2 and ci == 32 and co % 8 == 0 and co <= 64 and not fits:
        # tiles of one image's output, at most 128 pixels each, all channels: from 256 workgroups up
        per_image = ceil_div(ceil_div(h, 2) * ceil_div(w, 2), 128)
        assert out[4] == 256 and max(256, b * per_image) <= out[1] <= round8(2 * b * per_image), (shape, out)
        fits = [(128, 64)]
    if st == 1 and ci % 64 == 0 and co % 8 == 0 and not fits:
        # tiles of one image's output, at most 256 pixels each, times blocks of 64 channels: at least as
        # many as the pixels need, no image shares a tile, and the path is only taken from 128 workgroups up
        per_image = ceil_div(h * w, 256)
        assert out[4] == 256 and out[1] >= max(128, b * per_image * ceil_div(co, 64)), (shape, out)
        assert out[1] <= round8(2 * b * per_image * ceil_div(co, 64)), (shape, out)      # and not wastefully many
        fits = [(256, 64)]
    assert fits, (shape, out)
    assert out[1] * max(t[0] * t[1] for t in fits) >= pixels * co


# Tiles per image of the stride-1 kernel that keeps its input patch in LDS: th x tw output pixels, th * tw <= 256,
# (th + 2) * (tw + 2) <= 352, as few as cover the image.  Worked by hand:
#   208 x 208: 169 = 13 x 13 tiles of 16 x 16 (patch 18 x 18 = 324); 43264 / 256 = 169 is the least possible.
#   104 x 104: at least 43 (10816 / 256 = 42.25).  43 is prime and 44 = 4 x 11 = 2 x 22 would need a tile 26 high
#     (104 / 4) and 10 wide (104 / 11 rounded up) = 260 pixels, or 52 high: neither fits.  45 = 5 x 9: tiles of 21 x 12
#     (252 pixels, patch 23 x 14 = 322).
#   52 x 52: at least 11 (2704 / 256 = 10.6); 11 is prime: one row of 11 tiles would be 52 high and then at most 4 wide.
#     12 = 2 x 6: tiles of 26 x 9 (234 pixels, patch 28 x 11 = 308).
#   26 x 26: at least 3; 3 x 1: tiles of 9 x 26 (234 pixels, patch 11 x 28 = 308).
#   12 x 13: the whole image (156 pixels, patch 14 x 15 = 210).
#   100 x 90: at least 36 (9000 / 256 = 35.2); 6 x 6 tiles of 17 x 15 (255 pixels, patch 19 x 17 = 323).
@pytest.mark.parametrize("h,w,tiles", [(208, 208, 169), (104, 104, 45), (52, 52, 12), (26, 26, 3), (12, 13, 1), (100, 90, 36)])
def test_patch_kernel_tiles_per_image_worked_by_hand(h, w, tiles):
    batch = ceil_div(128, tiles)                                       # enough images for the path to be taken
    out = _probe("orc_conv3x3_probe", batch, h, w, 64, 64, 1)
    assert out[1:] == [round8(batch * tiles), 1, 1, 256, 1, 1]
    out = _probe("orc_conv3x3_probe", batch, h, w, 128, 136, 1)        # three blocks of 64 channels
    assert out[1] == round8(batch * tiles * 3)
    # one workgroup short of 128: the layer takes the other kernels (tiles of flattened pixels)
    if batch * tiles - tiles < 128 and batch > 1:
        out = _probe("orc_conv3x3_probe", batch - 1, h, w, 64, 64, 1)
        pixels = (batch - 1) * h * w
        assert out[1] in (round8(ceil_div(pixels, 256)), round8(ceil_div(pixels, 64)))


# The stride-2 kernel for 32 input channels: tiles of th x tw output pixels, th * tw <= 128, th + tw <= 30,
# (2 th + 1) * (2 tw + 1) <= 576.  Worked by hand:
#   208 x 208 (the net's second layer at 416 x 416): 338 = 26 x 13 tiles of 8 x 16 (patch 17 x 33 = 561);
#     43264 / 128 = 338 is the least possible.
#   75 x 76: at least 45 (5700 / 128 = 44.5).  45 = 9 x 5 needs tiles 9 high (75 / 9 rounded up) and 16 wide
#     (76 / 5 rounded up) = 144 pixels, 5 x 9 tiles 15 x 9 = 135, 3 x 15 tiles 25 x 6 = 150, 15 x 3 tiles 5 x 26 = 130:
#     none fits; 46 = 2 x 23 and 47 fit no better (tiles 38 or 75 high); 48 = 8 x 6: tiles of 10 x 13 = 130 do not fit,
#     6 x 8: 13 x 10 = 130 neither, 4 x 12: 19 x 7 = 133, 12 x 4: 7 x 19 = 133, 3 x 16: 25 x 5 = 125 pixels (25 + 5 = 30) with a patch of
#     51 x 11 = 561: fits.  So 48.
@pytest.mark.parametrize("h,w,tiles", [(416, 416, 338), (150, 151, 48)])
def test_stride2_kernel_tiles_per_image_worked_by_hand(h, w, tiles):
    batch = ceil_div(256, tiles)
    out = _probe("orc_conv3x3_probe", batch, h, w, 32, 64, 2)
    assert out[1:] == [round8(batch * tiles), 1, 1, 256, 1, 1]
    assert _probe("orc_conv3x3_probe", batch, h, w, 32, 40, 2)[1] == round8(batch * tiles)     # all channels in one workgroup
    # more than 64 channels: the ring kernel, 128 pixels x 128 channels per workgroup
    assert _probe("orc_conv3x3_probe", 8, h, w, 32, 136, 2)[1] == round8(ceil_div(8 * ceil_div(h, 2) * ceil_div(w, 2), 128) * 2)
    # 36864 (patch) + 36864 (filter) + 2304 (table) = 76032 bytes of LDS: two per CU
    assert (160 * 1024) // (576 * 64 + 64 * 576 + 576 * 4) == 2
    assert _lib().orc_conv3x3_residency(*[U(x) for x in (batch, h, w, 32, 64, 2)]) == 2


def test_patch_kernel_residency_from_its_lds():
    # 352 patch pixels x 64 channels x 2 bytes + four weight tiles of 64 x 64 x 2 bytes = 77824 bytes: two per CU
    assert (160 * 1024) // (352 * 128 + 4 * 8192) == 2
    assert _lib().orc_conv3x3_residency(*[U(x) for x in (8, 104, 104, 128, 128, 1)]) == 2


def test_net_geometry_is_its_largest_launch():
    net = [(3, 32, 1), (32, 64, 2), (64, 64, 1), (64, 128, 2), (128, 128, 1), (128, 256, 2), (256, 256, 1),
           (256, 512, 2), (512, 512, 1), (512, 512, 2)]
    for batch in (1, 2, 4, 8):
        out = _cnn_probe(net, batch, 416, 416)
        per_layer, h = [], 416
        for ci, co, st in net:
            per_layer.append(_probe("orc_conv3x3_probe", batch, h, h, ci, co, st))
            h = ceil_div(h, st)
        # (a small deep layer may be split further inside a chain, so the chain's largest launch is at
        # least the largest single-layer launch; the first layer has no launch of its own here: the
        # second layer's kernel computes it on the fly)
        assert out[1] * out[4] >= max(p[1] * p[4] for p in per_layer[1:])
        # the second layer: 208 x 208 output pixels per image in tiles of 8 x 16 = 338 * batch workgroups,
        # the third: 13 x 13 tiles of 16 x 16 per image = 169 * batch; at batch 1 a deeper, split layer has more
        assert per_layer[1][1:5] == [round8(338 * batch), 1, 1, 256] and per_layer[2][1] == round8(169 * batch)
        if batch >= 2:
            assert out[1:] == [round8(338 * batch), 1, 1, 256, 1, 1]
        # with the first layer alone (nothing behind it to compute it in) its own launch counts
        assert _cnn_probe(net[:1], batch, 416, 416)[1] == round8(676 * batch)


@pytest.mark.parametrize("n", [1, 100, 4096, 4097, 1 << 16, 1 << 20, (1 << 20) + 1, 1 << 22, 5000000])
def test_bfs_grid_is_one_workgroup_per_4096_vertices_within_8_and_512(n):
    out = _probe("orc_bfs_probe", n, 10)
    assert out[1:] == [min(512, max(8, round8(ceil_div(n, 4096)))), 1, 1, 512, 1, 1]
    if 8 * 4096 <= n <= 512 * 4096:
        assert out[1] * 4096 >= n


@pytest.mark.parametrize("n,iters", [(3, 1), (64, 10), (77, 3), (512, 20), (1024, 10), (2048, 100), (4096, 100), (4096, 4), (8192, 50),
                                     (16384, 50), (4100, 7), (1023, 5)])
def test_jacobi_grid_covers_the_interior(n, iters):
    out = _probe("orc_jacobi_probe", n, iters)
    assert out[4:] == [256, 1, 1] and out[0] == 8 * n * n
    waves = out[1] * 4
    if n % 4:
        # one column per thread, 8 rows per workgroup
        assert out[1] == round8(ceil_div(n, 256) * ceil_div(n - 2, 8))
    else:
        # a wave never produces more than 248 columns x (rows of its run): at most 248 x 8 cells per wave
        # for the window kernels; the streaming kernels produce 240 columns x a run of rows, and a run
        # is never longer than the whole interior
        most = 248 * 8 if not (n >= 2048 and iters >= 5) else 240 * (n - 2)
        assert waves * most >= (n - 2) * (n - 2)
        assert waves >= ceil_div(n - 2, 248)                        # at least one wave per column window


def test_configured_jacobi_launch_shapes():
    # 4096^2 x100 = 2 x 8 + 12 x 7 sweeps, streaming kernel: 18 strips of 240 columns (4096 = 256 + 16 * 240),
    # runs chosen so that the waves are one round of 2048: 2048 // 18 = 113 runs -> ceil(4094 / 113) = 37 rows
    # -> ceil(4094 / 37) = 111 runs -> 18 * 111 = 1998 waves -> 500 workgroups -> 504
    assert _probe("orc_jacobi_probe", 4096, 100)[1] == 504
    # 2048^2 x100 (the smallest grid that streams): 9 strips (2048 = 256 + 7.47 * 240), 2048 // 9 = 227 runs ->
    # ceil(2046 / 227) = 10 rows -> ceil(2046 / 10) = 205 runs -> 9 * 205 = 1845 waves -> 462 workgroups -> 464
    assert _probe("orc_jacobi_probe", 2048, 100)[1] == 464
    # 2044^2 x100: windows of 248 columns x 8 rows: (1 + ceil(1788 / 248)) x ceil(2042 / 8) = 9 x 256 waves = 576 workgroups
    assert _probe("orc_jacobi_probe", 2044, 100)[1] == 576
    # 512^2 x20 (the smoke mix): windows of 248 columns x 8 rows: 3 x 64 waves = 48 workgroups
    assert _probe("orc_jacobi_probe", 512, 20)[1] == 48


# ------------------------------------------------------------------ workgroups per CU from the CU's budgets
def wg_per_cu(lds_bytes, regs_per_lane, waves_per_wg):
    """What one CU holds: 160 KiB of LDS, 4 SIMDs each with 512 registers per lane (a wave's registers
    come in one piece from one SIMD), 32 wave slots."""
    by_lds = (160 * KIB) // lds_bytes if lds_bytes else 1 << 30
    by_regs = (4 * (512 // regs_per_lane)) // waves_per_wg
    by_slots = 32 // waves_per_wg
    return min(by_lds, by_regs, by_slots)


def test_residency_follows_from_lds_registers_and_wave_slots():
    lib = _lib()
    # fp32 GEMM, DMA kernels: LDS ring of 4 stages x (tile_m + tile_n) rows x 16 floats
    ring = lambda tm, tn, depth, size: 4 * (tm + tn) * depth * size
    assert ring(256, 256, 16, 4) == 128 * KIB and ring(128, 128, 16, 4) == 64 * KIB and ring(64, 64, 16, 4) == 32 * KIB
    #   256 x 256 tile: 4 waves of 128 x 128 -> 256 accumulator registers, 512 in all per lane
    assert lib.orc_gemm_f32_residency(U(4096), U(4096), U(4096)) == wg_per_cu(128 * KIB, 512, 4) == 1
    #   128 x 128 tile: 8 waves of 64 x 32 (64 registers)
    assert lib.orc_gemm_f32_residency(U(2048), U(2048), U(64)) == wg_per_cu(64 * KIB, 64, 8) == 2
    #   64 x 64 tile: 4 waves of one 32 x 32 block each (40 registers: the wave slots allow 8, LDS 5)
    assert lib.orc_gemm_f32_residency(U(256), U(256), U(256)) == wg_per_cu(32 * KIB, 40, 4) == 5
    #   register-staged kernel (k not a multiple of 16): two 16 KiB buffers, 8 waves per workgroup, 64 registers
    assert lib.orc_gemm_f32_residency(U(129), U(257), U(17)) == wg_per_cu(32 * KIB, 64, 8) == 4
    # bf16 GEMM: ring of 4 x (tm + tn) x 32 bf16
    assert ring(256, 256, 32, 2) == 128 * KIB
    assert lib.orc_gemm_bf16_residency(U(4096), U(4096), U(4096)) == wg_per_cu(128 * KIB, 512, 4) == 1
    assert lib.orc_gemm_bf16_residency(U(1024), U(1024), U(1024)) == wg_per_cu(64 * KIB, 116, 4) == 2
    #   register-staged (k not a multiple of 32): 4 waves of 211 registers -> two waves per SIMD; 56 KiB of LDS
    assert lib.orc_gemm_bf16_residency(U(129), U(257), U(17)) == wg_per_cu(56 * KIB, 211, 4) == 2
    # conv: ring of 4 x (pixels + channels) x depth bf16
    #   128 x 128 tiles, depth 32 (c_out > 64, enough tiles)
    assert lib.orc_conv3x3_residency(*[U(x) for x in (8, 104, 104, 128, 128, 1)]) == wg_per_cu(ring(128, 128, 32, 2), 111, 4) == 2
    #   256 x 64 tiles (c_out <= 64)
    assert ring(256, 64, 32, 2) == 80 * KIB
    assert lib.orc_conv3x3_residency(*[U(x) for x in (8, 416, 416, 32, 64, 2)]) == wg_per_cu(80 * KIB, 115, 4) == 2
    #   64 x 64 tiles, depth 64 split over four waves (c_in % 64 == 0, too few big tiles)
    assert lib.orc_conv3x3_residency(*[U(x) for x in (1, 104, 104, 128, 128, 1)]) == wg_per_cu(ring(64, 64, 64, 2), 174, 4) == 2
    #   64 x 64 tiles, depth 32, one wave per workgroup (c_in % 64 != 0)
    assert lib.orc_conv3x3_residency(*[U(x) for x in (1, 52, 52, 96, 72, 1)]) == wg_per_cu(ring(64, 64, 32, 2), 121, 1) == 5
    #   first layer (3 -> 32): three strips of 260 pixels x 4 bf16 + 256 x 32 bf16 of output staging
    assert 3 * 260 * 8 + 256 * 32 * 2 == 22624
    assert lib.orc_conv3x3_residency(*[U(x) for x in (1, 416, 416, 3, 32, 1)]) == wg_per_cu(22624, 72, 4) == 7
    #   (3 -> 64: twice the output staging)
    assert lib.orc_conv3x3_residency(*[U(x) for x in (2, 416, 416, 3, 64, 1)]) == wg_per_cu(3 * 260 * 8 + 256 * 64 * 2, 112, 4) == 4
    #   anything else: register-staged, 4 waves of up to 244 registers (two waves per SIMD), up to 72 KiB of LDS
    assert lib.orc_conv3x3_residency(*[U(x) for x in (1, 5, 6, 5, 7, 1)]) == wg_per_cu(72 * KIB, 244, 4) == 2
    # BFS level kernel: 8 waves of 120 registers; 29184 bytes of staging, plus the 128 KiB frontier
    # bitmap for graphs of up to 2^20 vertices (a bitmap of n bits in words, rounded up to 64 words)
    assert lib.orc_bfs_residency(U(1 << 20)) == wg_per_cu(29184 + 128 * KIB, 120, 8) == 1
    assert lib.orc_bfs_residency(U(1 << 19)) == wg_per_cu(29184 + 64 * KIB, 120, 8) == 1
    assert lib.orc_bfs_residency(U(1 << 18)) == wg_per_cu(29184 + 32 * KIB, 120, 8) == 2
    assert lib.orc_bfs_residency(U(1 << 16)) == wg_per_cu(29184 + 8 * KIB, 120, 8) == 2
    assert lib.orc_bfs_residency(U((1 << 20) + 1)) == wg_per_cu(29184, 120, 8) == 2
    # Jacobi: 4 waves per workgroup; one sweep per launch (n % 4 != 0): small kernels, the wave slots bind;
    # window kernels up to 168 registers (3 waves per SIMD); streaming kernels (n >= 2048) up to 224 (2)
    assert lib.orc_jacobi_residency(U(77)) == wg_per_cu(0, 11, 4) == 8
    assert lib.orc_jacobi_residency(U(2044)) == wg_per_cu(0, 168, 4) == 3
    assert lib.orc_jacobi_residency(U(2048)) == lib.orc_jacobi_residency(U(4096)) == wg_per_cu(0, 224, 4) == 2


def test_demands_of_the_mix16_kinds_follow_from_grid_and_residency():
    # Alg. 2's rule per CU: a task needs ceil(workgroups / workgroups per CU) CUs
    lib = _lib()
    dev = oracle.device(1 << 40, granule_cus=32)
    for probe, args, res in (("orc_gemm_f32_probe", (4096, 4096, 4096), lib.orc_gemm_f32_residency(U(4096), U(4096), U(4096))),
                             ("orc_jacobi_probe", (4096, 100), lib.orc_jacobi_residency(U(4096))),
                             ("orc_bfs_probe", (1 << 20, 1 << 24), lib.orc_bfs_residency(U(1 << 20)))):
        out = _probe(probe, *args)
        cus = ceil_div(out[1], res)
        assert 224 < cus <= 256
        assert oracle.demand(dev, out[1:4], out[4:7], res)[0] == ceil_div(cus, 32) == 8
