"""The residency facts the probes pass to the scheduler, against what the compiler reports for the
kernels as they are compiled for gfx950 (registers per lane, static LDS, waves per SIMD).

Sec. II-A of the paper: the hardware places thread blocks until a resource of the SM runs out.
Here: a CU holds 160 KiB of LDS, 32 wave slots, and per SIMD as many waves as the compiler's
occupancy figure says (512 registers per lane shared by the waves of a SIMD).  The test compiles
each kernel file once with the compiler's resource remarks (host-side work: nothing runs on a GPU)
and derives the workgroups per CU of every kernel variant from that report, the LDS ring the
launch adds, and the waves per workgroup; mgb_*_residency and the checker must both say the same
for a shape that selects the variant."""
import ctypes as C
import os
import re
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

import oracle
import paper_2107_08538_amd as mgb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2107_08538_amd", "csrc")
U = C.c_uint64
KIB = 1024


def _report(name):
    cmd = ["hipcc", "-O3", "-std=c++17", "--offload-arch=gfx950", "-x", "hip", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Rpass-analysis=kernel-resource-usage", "-c", os.path.join(CSRC, name), "-o", os.devnull]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-3000:]
    out, cur = {}, None
    for line in r.stderr.splitlines():
        m = re.search(r"remark:\s+(Function Name|VGPRs|AGPRs|Occupancy \[waves/SIMD\]|LDS Size \[bytes/block\]):\s+(\S+)", line)
        if not m:
            continue
        key, val = m.group(1), m.group(2)
        if key == "Function Name":
            cur = out.setdefault(val, {})
        elif cur is not None:
            cur[key.split(" ")[0]] = int(val)
    return out


@pytest.fixture(scope="module")
def reports():
    if shutil.which("hipcc") is None:
        pytest.skip("hipcc not found")
    names = ["gemm_f32.hip", "gemm_bf16.hip", "conv3x3.hip", "bfs.hip", "jacobi.hip"]
    with ThreadPoolExecutor(max_workers=5) as ex:
        reps = list(ex.map(_report, names))
    merged = {}
    for r in reps:
        merged.update(r)
    return merged


def _kernel(reports, *fragments):
    hits = [(n, r) for n, r in reports.items() if all(f in n for f in fragments)]
    assert len(hits) == 1, (fragments, [n for n, _ in hits])
    return hits[0][1]


def wg_per_cu(rep, waves_per_wg, ring_bytes=0):
    lds = rep["LDS"] + ring_bytes
    lds = -(-lds // 512) * 512                                  # LDS is handed out in pieces of 512 bytes
    by_lds = (160 * KIB) // lds if lds else 1 << 30
    by_regs = 4 * rep["Occupancy"] // waves_per_wg
    by_slots = 32 // waves_per_wg
    return max(1, min(by_lds, by_regs, by_slots))


def ring(rows, depth, size):
    return 4 * rows * depth * size                              # four stages


def test_fp32_gemm_variants(reports):
    lib = oracle.lib()
    lib.orc_gemm_f32_residency.restype = C.c_uint64
    # template arguments: waves along m, waves along n, 32 x 32 blocks per wave along m, along n
    cases = [((4096, 4096, 4096), _kernel(reports, "gemm_f32_dma_kernel", "ILj2ELj2ELj4ELj4E"), 4, ring(512, 16, 4)),   # 256 x 256
             ((2048, 2048, 64), _kernel(reports, "gemm_f32_dma_kernel", "ILj2ELj4ELj2ELj1E"), 8, ring(256, 16, 4)),      # 128 x 128
             ((256, 256, 256), _kernel(reports, "gemm_f32_dma_kernel", "ILj2ELj2ELj1ELj1E"), 4, ring(128, 16, 4)),       # 64 x 64
             ((129, 257, 17), _kernel(reports, "gemm_f32_kernel", "ILb1E"), 8, 0)]
    want = []
    for shape, rep, waves, ring_bytes in cases:
        w = wg_per_cu(rep, waves, ring_bytes)
        want.append(w)
        assert mgb.mgb_gemm_f32_residency(*shape) == w == lib.orc_gemm_f32_residency(*[U(x) for x in shape]), (shape, rep)
    assert want == [1, 2, 5, 4]


def test_bf16_gemm_variants(reports):
    lib = oracle.lib()
    lib.orc_gemm_bf16_residency.restype = C.c_uint64
    def a64(tile):                                              # A: three stages 64 deep; B: four stages 32 deep
        return 3 * tile * 64 * 2 + 4 * 32 * tile * 2
    cases = [((4096, 4096, 4064), _kernel(reports, "gemm_bf16_dma_kernel", "ILj4E"), 4, ring(512, 32, 2)),
             ((1024, 1024, 992), _kernel(reports, "gemm_bf16_dma_kernel", "ILj2E"), 4, ring(256, 32, 2)),
             ((4096, 4096, 4096), _kernel(reports, "gemm_bf16_dma_a64_kernel", "ILj4E"), 4, a64(256)),
             ((1024, 1024, 1024), _kernel(reports, "gemm_bf16_dma_a64_kernel", "ILj2E"), 4, a64(128)),
             ((129, 257, 17), _kernel(reports, "gemm_bf16_kernel", "ILb0E"), 4, 0)]
    want = []
    for shape, rep, waves, ring_bytes in cases:
        w = wg_per_cu(rep, waves, ring_bytes)
        want.append(w)
        assert mgb.mgb_gemm_bf16_residency(*shape) == w == lib.orc_gemm_bf16_residency(*[U(x) for x in shape]), (shape, rep)
    assert want == [1, 2, 1, 2, 2]


def test_conv_variants(reports):
    lib = oracle.lib()
    lib.orc_conv3x3_residency.restype = C.c_uint64
    cases = [((8, 104, 104, 96, 128, 1), _kernel(reports, "conv3x3_dma_kernel", "ILj2ELj2E"), 4, ring(256, 32, 2)),    # 128 x 128
             ((8, 416, 416, 32, 64, 1), _kernel(reports, "conv3x3_dma_kernel", "ILj4ELj1E"), 4, ring(320, 32, 2)),     # 256 x 64
             # stride 2 from 32 channels: patch of 576 pixels x 64 bytes, the filter of 64 channels, a table of 576 words
             ((8, 416, 416, 32, 64, 2), _kernel(reports, "conv3x3_s2c32_kernel", "ILb0E"), 4, 576 * 64 + 64 * 576 + 576 * 4),
             # the same tiles fed by two stages of depth 64 (c_in % 64 == 0; stride 2: stride 1 takes the patch kernel)
             ((8, 208, 208, 64, 128, 2), _kernel(reports, "conv3x3_dma64_kernel", "ILj2ELj2E"), 4, ring(256, 64, 2) // 2),
             ((8, 416, 416, 64, 64, 2), _kernel(reports, "conv3x3_dma64_kernel", "ILj4ELj1E"), 4, ring(320, 64, 2) // 2),
             # stride 1, c_in % 64 == 0: patch of 352 pixels x 128 bytes and four weight tiles of 8 KiB
             ((8, 104, 104, 128, 128, 1), _kernel(reports, "conv3x3_patch_kernel"), 4, 352 * 128 + 4 * 8 * KIB),
             ((1, 104, 104, 128, 128, 1), _kernel(reports, "conv3x3_dma_ksplit_kernel"), 4, ring(128, 64, 2)),         # 64 x 64, depth 64
             ((1, 52, 52, 96, 72, 1), _kernel(reports, "conv3x3_dma_kernel", "ILj1ELj1E"), 1, ring(128, 32, 2)),       # 64 x 64, one wave
             ((1, 416, 416, 3, 32, 1), _kernel(reports, "conv3x3_c3_kernel", "ILj1E"), 4, 0),
             ((2, 416, 416, 3, 64, 1), _kernel(reports, "conv3x3_c3_kernel", "ILj2E"), 4, 0)]
    want = []
    for shape, rep, waves, ring_bytes in cases:
        w = wg_per_cu(rep, waves, ring_bytes)
        want.append(w)
        assert mgb.mgb_conv3x3_residency(*shape) == w == lib.orc_conv3x3_residency(*[U(x) for x in shape]), (shape, rep)
    assert want == [2, 2, 2, 2, 2, 2, 2, 5, 7, 4]
    # the same kernel computing the 3-channel first layer on the fly (inside a chain): the first layer's filter
    # (32 x 27 values) and 705 raw pixels of 8 bytes instead of the table
    fused = wg_per_cu(_kernel(reports, "conv3x3_s2c32_kernel", "ILb1E"), 4, 576 * 64 + 64 * 576 + 32 * 27 * 2 + 705 * 8)
    net = [(3, 32, 1), (32, 64, 2)]
    flat = (mgb.mgb_conv_layer * 2)(*[mgb.mgb_conv_layer(*L) for L in net])
    assert mgb.mgb_cnn_residency(flat, 2, 8, 416, 416) == fused == 2
    # the register-staged kernels (any other shape) are reported as 2 per CU: never more than they can hold
    for frag in ("ILj64ELb1E", "ILj64ELb0E", "ILj128ELb1E", "ILj128ELb0E"):
        assert wg_per_cu(_kernel(reports, "conv3x3_kernel", frag), 4) >= 2
    assert mgb.mgb_conv3x3_residency(1, 5, 6, 5, 7, 1) == 2


def test_bfs_and_jacobi_variants(reports):
    lib = oracle.lib()
    lib.orc_bfs_residency.restype = lib.orc_jacobi_residency.restype = C.c_uint64
    level = _kernel(reports, "bfs_level")
    for n, bitmap in ((1 << 20, 128 * KIB), (1 << 19, 64 * KIB), (1 << 18, 32 * KIB), (1 << 16, 8 * KIB), ((1 << 20) + 1, 0), (1 << 22, 0)):
        w = wg_per_cu(level, 8, bitmap)
        assert mgb.mgb_bfs_residency(n) == w == lib.orc_bfs_residency(U(n)), n
    assert wg_per_cu(level, 8, 128 * KIB) == 1 and wg_per_cu(level, 8, 0) == 2
    # Jacobi: the residency of a grid size is that of the largest kernel its launches may use
    windows = min(wg_per_cu(_kernel(reports, "jacobi_sweeps", "ILj%dE" % t), 4) for t in (1, 2, 3, 4))
    streams = min(wg_per_cu(_kernel(reports, "jacobi_stream", "ILj%dE" % t), 4) for t in (5, 6, 7, 8))
    one = wg_per_cu(_kernel(reports, "jacobi_sweep_v1"), 4)
    assert (windows, streams, one) == (3, 2, 8)
    for n, w in ((2044, windows), (512, windows), (2048, min(windows, streams)), (4096, min(windows, streams)), (16384, min(windows, streams)), (77, one)):
        assert mgb.mgb_jacobi_residency(n) == w == lib.orc_jacobi_residency(U(n)), n


# ---- what the main loops of the MFMA kernels issue between their MFMAs -----------------------------
#
# With one wave per SIMD a vector-ALU instruction between two MFMAs holds the matrix pipe up for ~14
# clocks and a load with a 64-bit vector address for 10-17 more, while scalar instructions, LDS reads
# with immediate offsets and buffer loads with scalar offsets are free.  The ring kernels are written so
# that their main loops hold none of the former; this reads the compiler's assembly to keep it so.

def _assembly(name):
    cmd = ["hipcc", "-O3", "-std=c++17", "--offload-arch=gfx950", "-x", "hip", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Wno-inline-asm", "-S", "--cuda-device-only", os.path.join(CSRC, name), "-o", "-"]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-3000:]
    return r.stdout.split("\n")


@pytest.fixture(scope="module")
def assemblies():
    if shutil.which("hipcc") is None:
        pytest.skip("hipcc not found")
    names = ["gemm_f32.hip", "gemm_bf16.hip", "conv3x3.hip"]
    with ThreadPoolExecutor(max_workers=3) as ex:
        return dict(zip(names, ex.map(_assembly, names)))


def _main_loop(lines, fragment):
    """Instruction names from the loop header that is followed by the most MFMAs to the kernel's last MFMA."""
    start = [i for i, l in enumerate(lines) if fragment in l and "@function" in l]
    assert len(start) == 1, (fragment, len(start))
    end = [i for i, l in enumerate(lines) if i > start[0] and l.strip().startswith(".size") and fragment in l][0]
    body = lines[start[0]:end]
    mfma = [i for i, l in enumerate(body) if "v_mfma" in l]
    headers = [i for i, l in enumerate(body) if "Loop Header" in l and i < mfma[-1]]
    assert headers, fragment
    h = max(headers, key=lambda i: sum(1 for j in mfma if i < j < i + 3000))
    return [l.split()[0] for l in body[h:mfma[-1] + 1]
            if l.startswith("\t") and l.strip() and not l.strip().startswith((";", "."))]


@pytest.mark.parametrize("source,fragment,mfmas,max_valu,kinds", [
    # four ring stages per pass; the compiler recomputes a few addresses at the loop header
    ("gemm_f32.hip", "gemm_f32_dma_kernelILj2ELj2ELj4ELj4E", 512, 8, {"v_add_u32_e32"}),
    ("gemm_f32.hip", "gemm_f32_dma_kernelILj2ELj4ELj2ELj1E", 64, 8, {"v_add_u32_e32"}),
    # twelve combinations of A and B stage per pass
    ("gemm_bf16.hip", "gemm_bf16_dma_a64_kernelILj4E", 384, 8, {"v_add_u32_e32"}),
    ("gemm_bf16.hip", "gemm_bf16_dma_a64_kernelILj2E", 96, 8, {"v_add_u32_e32"}),
    # conv: a new filter tap selects each lane's offsets (and, compare, select per DMA instruction), nothing per tile
    ("conv3x3.hip", "conv3x3_dma64_kernelILj2ELj2E", 32, 16, {"v_and_b32_e32", "v_cmp_eq_u32_e32", "v_cndmask_b32_e32", "v_mov_b32_e32"}),
    ("conv3x3.hip", "conv3x3_dma_ksplit_kernel", 16, 24, {"v_and_b32_e32", "v_cmp_eq_u32_e32", "v_cndmask_b32_e32", "v_mov_b32_e32"}),
])
def test_main_loops_hold_no_vector_arithmetic_between_mfmas(assemblies, source, fragment, mfmas, max_valu, kinds):
    ops = _main_loop(assemblies[source], fragment)
    assert sum(1 for o in ops if "v_mfma" in o) == mfmas, (fragment, sum(1 for o in ops if "v_mfma" in o))
    valu = [o for o in ops if o.startswith("v_") and "mfma" not in o and not o.startswith("v_accvgpr")]
    assert len(valu) <= max_valu and set(valu) <= kinds, (fragment, sorted(set(valu)), len(valu))
    assert not [o for o in ops if o.startswith(("global_load", "flat_load"))], fragment     # DMA: buffer loads only
    assert [o for o in ops if o.startswith("buffer_load")], fragment
