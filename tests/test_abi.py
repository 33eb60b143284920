"""CPU checks of the boundary: the built library loads and exports every function that
include/gemm_f32.h declares, and the host-side queries that need no GPU answer correctly."""
from __future__ import annotations

import os
import re

from paper_2002_02268_amd import binding

INCLUDE = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")


def declared_functions():
    names = []
    for header in sorted(os.listdir(INCLUDE)):
        text = open(os.path.join(INCLUDE, header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b([a-z_0-9]+)\s*\([^;{]*\)\s*;", text)
    return sorted(set(names))


def test_header_declares_the_expected_entry_points():
    names = declared_functions()
    for must in ("gemm_f32", "gemm_f32_batched", "pack_b", "pack_b_size", "gemm_f32_packed",
                 "gemm_f32_set_stream", "gemm_f32_strerror", "gemm_f32_last_hip_error",
                 "gemm_f32_ladder", "gemm_f32_ladder_levels", "gemm_f32_ladder_name"):
        assert must in names


def test_library_exports_every_declared_symbol():
    lib = binding.lib()
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared in gemm_f32.h but not exported"
        assert name in binding.SYMBOLS, f"{name} has no Python binding signature"


def test_host_only_queries():
    lib = binding.lib()
    P = binding.pack_b_panel_width()
    assert P > 0 and P % 4 == 0
    assert binding.pack_b_size(0, 5) == 0 and binding.pack_b_size(5, 0) == 0
    assert binding.pack_b_size(1, 1) == P * 4
    assert binding.pack_b_size(P + 1, 7) == 2 * 7 * P * 4
    assert lib.gemm_f32_strerror(0) == b"ok"
    assert lib.gemm_f32_strerror(-99) == b"unknown status"
    assert lib.gemm_f32_last_hip_error() == 0
    # argument validation happens before anything touches a device
    assert lib.gemm_f32(-1, 1, 1, None, 1, None, 1, None, 1, 0) == -1
    assert lib.gemm_f32(4, 4, 4, None, 4, None, 4, None, 4, 0) == -2
    assert lib.gemm_f32(0, 4, 4, None, 4, None, 4, None, 4, 0) == 0
    assert lib.gemm_f32_batched(0, 4, 4, 4, None, 4, 16, None, 4, 16, None, 4, 16, 0) == 0
    assert binding.variant_name(4096, 4096, 4096).startswith("t128x128")
    assert binding.variant_name(8192, 8192, 8192).startswith("t256x256")     # operands beyond the memory-side cache
    assert "/a4" in binding.variant_name(1000, 1030, 999)


def test_large_shapes_with_a_partly_filled_last_round_keep_their_measured_tiles():
    """Choices the timing audit of large shapes established (the split of a last round is priced by what its pieces
    take beyond the window in which whole tiles end; a tile alone on its compute unit gets no such window): the
    256 x 256 tile with 88 tail tiles in two pieces took 1377 us on the first shape, the 128 x 128 tile 1245."""
    assert binding.variant_name(2048, 11008, 4096, transB=True) == "t128x128x16/nt/a16/tail96x2"
    assert binding.variant_name(6144, 6144, 6144) == "t128x128x16/nn/a16"
    assert binding.variant_name(4352, 4352, 4096).startswith("t64x128x32/nn/a16")     # first of the two orientations
    assert binding.variant_name(4224, 4224, 4096) == "t128x128x16/nn/a16/tail65x3"
    assert binding.variant_name(512, 4096, 11008, transB=True).startswith("t64x128x32")   # not 512 co-resident 64 x 64 tiles


def test_ladder_host_queries():
    assert binding.gemm_f32_ladder_levels() == 7
    names = [binding.gemm_f32_ladder_name(i) for i in range(7)]
    assert names == ["baseline", "blocking", "vectorization", "loop permutation", "array packing",
                     "cache blocks", "parallel"]
    assert binding.gemm_f32_ladder_name(7) == "invalid"
    lib = binding.lib()
    assert lib.gemm_f32_ladder(9, 4, 4, 4, None, 4, None, 4, None, None, 4) == -1
    assert lib.gemm_f32_ladder(0, 4, 4, 4, None, 4, None, 4, None, None, 4) == -2
    assert lib.gemm_f32_ladder(0, 0, 4, 4, None, 4, None, 4, None, None, 4) == 0


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = os.path.dirname(INCLUDE)
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_traffic_figures_are_dropped_when_the_kernel_sources_change():
    """bench.py reports HBM traffic only while the hash of the kernel sources matches the one the
    counters were taken with."""
    import importlib.util
    root = os.path.dirname(INCLUDE)
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(root, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    current = bench.kernel_sources_sha256()
    saved = bench.TRAFFIC["sources_sha256"]
    try:
        bench.TRAFFIC["sources_sha256"] = current
        t = bench.traffic_bytes("square4096")
        # between 1x and 6x the compulsory bytes (128 x 128 tiles: each of the eight L2 caches asks for its rows of A
        # and columns of B about six times over)
        assert t is not None and 4 * 3 * 4096 * 4096 <= t < 6 * 4 * 3 * 4096 * 4096
        bench.TRAFFIC["sources_sha256"] = "0" * 64
        assert bench.traffic_bytes("square4096") is None
        # ... and only while the dispatch still runs the variant they were taken on
        bench.TRAFFIC["sources_sha256"] = current
        variant = bench.TRAFFIC["square4096"]["variant"]
        assert variant == bench.workload_variant("square4096")
        bench.TRAFFIC["square4096"]["variant"] = "t256x256x16/nn/a16"
        assert bench.traffic_bytes("square4096") is None
        bench.TRAFFIC["square4096"]["variant"] = variant
    finally:
        bench.TRAFFIC["sources_sha256"] = saved


def test_dispatch_choices_for_the_benchmark_workloads():
    """The tile and split the cost model takes for the workloads the benchmark times (a host computation;
    pinned so that a change of the model's constants shows up here and not only as a slower benchmark)."""
    from paper_2002_02268_amd import synth
    want = {"square4096": "t128x128x16/nn/a16", "square1024": "t64x64x64/nn/a16", "transb2048": "t128x128x16/nt/a16",
            "ragged": "t64x64x64/nn/a4/strip6", "skinny8192": "t32x32x64k4/nn/a16",
            "wide8192": "t32x32x64k4/nt/a16"}
    for name, variant in want.items():
        w = synth.WORKLOADS[name]
        assert binding.variant_name(w["M"], w["N"], w["K"], transB=w["transB"]) == variant, name
    # wide outputs never take the 128 x 32 and 32 x 128 tiles; outputs no wider than 32 always take a 32-wide
    # tile: the one whose waves share the slabs where the long operand has k contiguous and needs no
    # element-wise masks
    narrow = ("t128x32x32", "t32x128x32")
    for M, N, K in [(1024, 1024, 1024), (300, 300, 300), (128, 128, 8192), (2048, 64, 2048), (64, 4096, 512)]:
        assert not binding.variant_name(M, N, K).startswith(narrow), (M, N, K)
    # outputs of a few hundred 32 x 32 blocks take the shared-slab tile and need no K split; large ones do not
    for M, N, K in [(640, 640, 1024), (512, 512, 4096), (300, 300, 300), (2048, 256, 1024)]:
        tile, layout, align = binding.variant_name(M, N, K).split("/")
        assert tile in ("t32x32x64k4", "t64x32x64k4", "t32x64x64k4") and (layout, align) == ("nn", "a16"), (M, N, K)
    for M, N, K in [(2048, 2048, 2048), (1280, 1280, 1280), (4096, 4096, 4096)]:
        assert "k4" not in binding.variant_name(M, N, K), (M, N, K)
    assert binding.variant_name(4096, 32, 4096).startswith("t32x32x64k4")
    assert binding.variant_name(8192, 8, 8192).startswith("t128x32x32")            # B stored K x 8: masked element-wise
    assert binding.variant_name(8192, 8, 8192, transB=True).startswith("t32x32x64k4")
    assert binding.variant_name(3000, 17, 1000).startswith("t128x32x32")
    assert binding.variant_name(5000, 20, 999, lda=999).startswith("t128x32x32")
    assert binding.variant_name(32, 4096, 4096).startswith("t32x32x64k4")
    for M, N, K in [(32, 4096, 4096), (1, 8192, 8192), (16, 11008, 4096)]:
        assert binding.variant_name(M, N, K, transB=True).startswith("t32x32x64k4"), (M, N, K)
    # at most 4 rows or columns, k-contiguous operands, a long operand of at least 160 MB too short for 256
    # blocks: the vector-unit kernel; otherwise the tiles
    assert binding.variant_name(4, 4096, 11008, transB=True) == "thin4x4/nt"
    assert binding.variant_name(4096, 2, 14336, transB=True) == "thin2x4/nt"
    for M, N, K in [(4, 4096, 4096), (4, 4096, 8192), (5, 4096, 11008), (4, 8192, 8192)]:
        assert not binding.variant_name(M, N, K, transB=True).startswith("thin"), (M, N, K)
    assert not binding.variant_name(4, 4096, 11008).startswith("thin")              # B stored K x N


def test_block_tails_are_planned_only_for_tiles_that_have_the_block_kernel():
    """The last round is cut into 32 x 32 blocks only for tile shapes whose kernel contains the block
    path (four waves that each own blocks); the tiles whose waves share the slabs split it along K."""
    import os
    import random
    rng = random.Random(5)
    with_blocks = {"t64x64x32", "t64x64x64", "t128x64x32", "t64x128x32", "t128x32x32", "t32x128x32"}
    try:
        for tile in range(13):
            binding.set_test_hooks(force_tile=tile)
            for _ in range(400):
                M, N, K = rng.randint(1, 3000), rng.randint(1, 3000), rng.randint(1, 5000)
                name = binding.variant_name(M, N, K, transB=rng.random() < 0.5)
                if "/quad" in name:
                    assert name.split("/")[0] in with_blocks, (M, N, K, name)
    finally:
        binding.set_test_hooks(force_tile=None)


def test_planning_from_many_host_threads_agrees_with_one_thread():
    """The dispatch's planning (cost model, its per-thread cache of choices, the per-thread name buffer) run
    from eight host threads at once on the same seeded shapes gives every thread the single-threaded answers."""
    import random
    import threading
    binding.set_test_hooks()
    rng = random.Random(17)
    shapes = [(rng.randint(1, 5000), rng.randint(1, 5000), rng.randint(1, 20000), rng.random() < 0.5) for _ in range(300)]
    want = [binding.variant_name(M, N, K, transB=t) for (M, N, K, t) in shapes]
    results, errors = {}, []

    def run(tid):
        try:
            order = list(range(len(shapes)))
            random.Random(tid).shuffle(order)
            got = {}
            for _ in range(3):
                for i in order:
                    M, N, K, t = shapes[i]
                    got[i] = binding.variant_name(M, N, K, transB=t)
            results[tid] = [got[i] for i in range(len(shapes))]
        except Exception as e:                      # pragma: no cover
            errors.append(e)

    threads = [threading.Thread(target=run, args=(tid,)) for tid in range(8)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors
    for tid in range(8):
        assert results[tid] == want


def test_test_hooks_validate_and_reset():
    lib = binding.lib()
    binding.set_test_hooks(force_tile=3)
    assert binding.variant_name(4096, 4096, 4096).startswith("t64x64x64")
    binding.set_test_hooks(force_tile=None, force_split=4)
    assert binding.variant_name(512, 512, 4096).endswith("splitk4")
    binding.set_test_hooks()
    assert binding.variant_name(4096, 4096, 4096).startswith("t128x128x16")
    bad = binding.HookSettings(force_tile=13)
    import ctypes
    assert lib.gemm_f32_set_test_hooks(ctypes.byref(bad)) == -1
    assert lib.gemm_f32_set_test_hooks(None) == 0
    # the environment is not a hook any more
    import os
    os.environ["GEMMF32_FORCE_TILE"] = "3"
    try:
        assert binding.variant_name(4096, 4096, 4096).startswith("t128x128x16")
    finally:
        os.environ.pop("GEMMF32_FORCE_TILE")
    assert lib.gemm_f32_noalloc_scratch_bytes() == 32 << 20
    assert lib.gemm_f32_strerror(-6).decode().startswith("the product needs more scratch")


def test_strip_is_weighed_against_the_edge_tile_column():
    """The last few columns of C go to the strip workgroups where that saves a round of tiles (or a split
    one), and stay an edge tile column where that column fits the last round anyway; the hooks force either."""
    import ctypes
    lib = binding.lib()
    binding.set_test_hooks()
    assert binding.variant_name(1000, 1030, 999).endswith("/strip6")            # 16 x 16 tiles + 6 columns: 272 tiles otherwise
    assert binding.variant_name(4096, 4100, 4096).endswith("/strip4")
    assert "/strip" not in binding.variant_name(700, 1286, 2000)                # 11 x 21 = 231 tiles: one round either way
    try:
        binding.set_test_hooks(force_strip=True, force_tile=3)
        assert binding.variant_name(700, 1286, 2000).endswith("/strip6")
        binding.set_test_hooks(force_strip=None, no_strip=True, force_tile=None)
        assert "/strip" not in binding.variant_name(1000, 1030, 999)
        # a strip needs 32-bit offsets along a row of A and over a chunk of B stored K x N
        binding.set_test_hooks()
        for rows, wait, ok in ((3, 0, False), (8, 0, False), (2, 66, False), (4, 65, True), (0, 0, True)):
            h = binding.HookSettings(force_tile=-1, strip_rows=rows, strip_wait=wait)
            assert (lib.gemm_f32_set_test_hooks(ctypes.byref(h)) == 0) == ok, (rows, wait)
    finally:
        binding.set_test_hooks()


def test_planning_an_empty_sum_over_many_tiles():
    """K = 0 with more tiles than one round and a remainder: the plan of the split last round has nothing to
    cut (this divided by zero once)."""
    for M, N in [(5000, 4000), (1000, 1030), (4100, 4100)]:
        name = binding.variant_name(M, N, 0)
        assert name not in ("invalid", "empty") and "/tail" not in name and "/quad" not in name, name
