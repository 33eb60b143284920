"""The strategy layer (include/elevate.h), host side only.

Pins: the combinators and traversals against the behaviour Section 3 of the paper states for them
(on small terms worked out by hand), the map-fusion style example of Section 3.5 (where `one` and
`body`/`argument` land), the doubly transposed matrix of Section 4 (the printed result and the
printed count of 12 rule applications, tests/golden/fsmooth_double_transpose.txt), tiling as split
plus interchange (Section 6.3), and the lowering of scheduled nests to kernel configurations."""
from __future__ import annotations

import os

import pytest

from paper_2002_02268_amd import binding as b

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "fsmooth_double_transpose.txt")
RULES = "(lChoice buildGet lenBuild letPartialEval letApp funToLet)"


def rw(strategy, program):
    return b.elevate_rewrite(strategy, program)


# ---------------------------------------------------------------- Section 3.2 - 3.4: basics, combinators

def test_id_succeeds_and_fail_names_itself():
    assert rw("id", "(get (build n f) i)") == (0, "(get (build n f) i)", 0)
    assert rw("fail", "x") == (b.ELEVATE_FAILED, "fail", 0)


def test_a_rule_matches_only_the_root():
    assert rw("buildGet", "(get (build n f) i)") == (0, "(app f i)", 1)
    # the same redex one level down is out of reach of the bare rule (Section 3.5)
    assert rw("buildGet", "(length (get (build n f) i))") == (b.ELEVATE_FAILED, "buildGet", 0)
    assert rw("lenBuild", "(length (build n f))") == (0, "n", 1)


def test_seq_needs_both_and_lchoice_tries_the_second_on_the_original():
    p = "(length (build (get (build n f) i) g))"
    assert rw("(seq lenBuild buildGet)", p) == (0, "(app f i)", 2)
    assert rw("(seq buildGet lenBuild)", p)[0] == b.ELEVATE_FAILED
    assert rw("(seq lenBuild lenBuild)", p) == (b.ELEVATE_FAILED, "lenBuild", 1)
    assert rw("(lChoice buildGet lenBuild)", p) == (0, "(get (build n f) i)", 1)
    assert rw("(lChoice lenBuild buildGet)", p) == (0, "(get (build n f) i)", 1)
    assert rw("(lChoice buildGet buildGet)", p)[0] == b.ELEVATE_FAILED


def test_try_never_fails_and_repeat_runs_until_not_applicable():
    assert rw("(try buildGet)", "x") == (0, "x", 0)
    nested = "(length (build (length (build (length (build n f)) g)) h))"
    assert rw("(repeat lenBuild)", nested) == (0, "n", 3)
    assert rw("(repeat lenBuild)", "n") == (0, "n", 0)


# ---------------------------------------------------------------- Section 3.5 - 3.7: traversals

def test_all_one_some():
    p = "(pair (length (build a f)) (length (build c g)) z)"
    assert rw("(one lenBuild)", p) == (0, "(pair a (length (build c g)) z)", 1)          # leftmost match only
    assert rw("(some lenBuild)", p) == (0, "(pair a c z)", 2)
    assert rw("(all lenBuild)", p)[0] == b.ELEVATE_FAILED                                  # z does not match
    assert rw("(all lenBuild)", "(pair (length (build a f)) (length (build c g)))") == (0, "(pair a c)", 2)
    assert rw("(one lenBuild)", "(pair x y)")[0] == b.ELEVATE_FAILED
    assert rw("(some lenBuild)", "(pair x y)")[0] == b.ELEVATE_FAILED
    assert rw("(all lenBuild)", "x") == (0, "x", 0)                                       # no sub-expressions


def test_language_specific_traversals_address_one_position():
    """Section 3.6 on the three-maps shape: two redexes, `body` reaches the outer one and
    `body(argument(...))` the inner one."""
    p = "(fun xs (app (get (build n f) i) (get (build m g) j)))"
    assert rw("(body (function buildGet))", p) == (0, "(fun xs (app (app f i) (get (build m g) j)))", 1)
    assert rw("(body (argument buildGet))", p) == (0, "(fun xs (app (get (build n f) i) (app g j)))", 1)
    assert rw("(function buildGet)", p)[0] == b.ELEVATE_FAILED       # the root is a function, not an application
    assert rw("(body buildGet)", "(app f x)")[0] == b.ELEVATE_FAILED


def test_topdown_takes_the_outermost_and_bottomup_the_innermost_redex():
    p = "(length (build (length (build a f)) (fun i (length (build c g)))))"
    assert rw("(topDown lenBuild)", p) == (0, "(length (build a f))", 1)
    assert rw("(bottomUp lenBuild)", p) == (0, "(length (build a (fun i (length (build c g)))))", 1)
    assert rw("(topDown lenBuild)", "(get x y)")[0] == b.ELEVATE_FAILED
    assert rw("(bottomUp lenBuild)", "(get x y)")[0] == b.ELEVATE_FAILED


def test_tryall_applies_everywhere_bottom_up_and_never_fails():
    p = "(pair (length (build a f)) (get (build n (fun i (length (build c g)))) j))"
    code, out, steps = rw("(tryAll (lChoice lenBuild buildGet))", p)
    assert (code, out, steps) == (0, "(pair a (app (fun i c) j))", 3)
    assert rw("(tryAll lenBuild)", "(pair x y)") == (0, "(pair x y)", 0)


def test_alltopdown_and_allbottomup_insist_on_every_node():
    # a strategy that applies to every node: try(r)
    assert rw("(allTopDown (try lenBuild))", "(pair (length (build a f)) z)") == (0, "(pair a z)", 1)
    assert rw("(allBottomUp (try lenBuild))", "(length (build (length (build a f)) g))") == (0, "a", 2)
    assert rw("(allTopDown lenBuild)", "(length (build a f))") == (0, "a", 1)            # an atom has no sub-terms
    assert rw("(allTopDown lenBuild)", "(length (build (pair x y) f))")[0] == b.ELEVATE_FAILED   # x does not match


def test_normalize_reaches_a_form_where_the_rule_applies_nowhere():
    p = "(pair (length (build (length (build a f)) g)) (fun i (length (build c h))))"
    code, out, steps = rw("(normalize lenBuild)", p)
    assert (code, out, steps) == (0, "(pair a (fun i c))", 3)
    assert rw("(topDown lenBuild)", out)[0] == b.ELEVATE_FAILED


def test_non_terminating_strategy_is_cut_off():
    # the paper's own example of a non-terminating normal form uses the always-applicable id; a
    # rule that swaps two loops forever is the same thing made of a rule, and is what the limit is for
    nest = "(loop M 4 seq (loop N 4 seq mac))"
    code, out, steps = rw("(repeat interchange)", nest)
    assert code == b.ELEVATE_ELIMIT and steps == 100000


# ---------------------------------------------------------------- Section 4: the doubly transposed matrix

def load_golden():
    vals = {}
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            key, _, rest = line.strip().partition(" ")
            vals[key] = rest
    return vals


def test_double_transpose_rewrites_to_the_program_without_transposition_in_12_steps():
    g = load_golden()
    code, out, steps, trace = b.elevate_rewrite(f"(normalize {RULES})", g["input"], trace=True)
    assert code == 0
    assert b.elevate_alpha_equal(out, g["output"]) == 1, out
    assert steps == int(g["steps"]) == 12
    lines = trace.strip().split("\n")
    assert len(lines) == 12
    used = [ln.split(":")[0] for ln in lines]
    assert used[0] == "letPartialEval"                   # the binding of MT is inlined first (top-down)
    assert set(used) == {"letPartialEval", "buildGet", "funToLet", "lenBuild"}
    # the result is a normal form of every rule
    assert rw(f"(topDown {RULES})", out)[0] == b.ELEVATE_FAILED


def test_rewrite_trace_is_deterministic():
    g = load_golden()
    runs = {b.elevate_rewrite(f"(normalize {RULES})", g["input"], trace=True) for _ in range(5)}
    assert len(runs) == 1


def test_substitution_avoids_capture():
    # let i = j in (fun j -> M[j][i]): the bound j must not capture the free j being substituted
    code, out, _ = rw("letPartialEval", "(let i j (fun j (get (get M j) i)))")
    assert code == 0
    assert b.elevate_alpha_equal(out, "(fun k (get (get M k) j))") == 1
    assert b.elevate_alpha_equal(out, "(fun j (get (get M j) j))") == 0
    # shadowing: the inner binding of x hides the outer one
    assert rw("letPartialEval", "(let x a (fun x (get x 0)))")[1] == "(fun x (get x 0))"
    assert rw("letPartialEval", "(let x a (let y (get x 0) (get y x)))")[1] == "(let y (get a 0) (get y a))"
    # letApp keeps the argument's free variable out of the binding's scope
    code, out, _ = rw("letApp", "(app (let x a (fun y (get y x))) x)")
    assert code == 0 and b.elevate_alpha_equal(out, "(let z a (app (fun y (get y z)) x))") == 1


def test_alpha_equality():
    assert b.elevate_alpha_equal("(fun i (fun j (get i j)))", "(fun a (fun b (get a b)))") == 1
    assert b.elevate_alpha_equal("(fun i (fun j (get i j)))", "(fun a (fun b (get b a)))") == 0
    assert b.elevate_alpha_equal("(fun i (get i k))", "(fun j (get j k))") == 1
    assert b.elevate_alpha_equal("(fun i (get i k))", "(fun k (get k k))") == 0
    assert b.elevate_alpha_equal("(let x a (get x x))", "(let y a (get y y))") == 1
    assert b.elevate_alpha_equal("(get x", "x") == b.ELEVATE_EPARSE


# ---------------------------------------------------------------- Section 6: scheduling rules on loop nests

NEST = "(loop M 1024 seq (loop N 512 seq (loop K 256 seq mac)))"


def test_split_is_loop_blocking_and_applies_only_where_valid():
    assert rw("(split M 128)", NEST)[1] == "(loop M 8 seq (loop M 128 seq (loop N 512 seq (loop K 256 seq mac))))"
    assert rw("(split N 128)", NEST)[0] == b.ELEVATE_FAILED                  # the root is the M loop
    assert rw("(topDown (split N 128))", NEST)[1] == \
        "(loop M 1024 seq (loop N 4 seq (loop N 128 seq (loop K 256 seq mac))))"
    assert rw("(split M 1024)", NEST)[0] == b.ELEVATE_FAILED                 # nothing to block
    assert rw("(split M 100)", NEST)[1].startswith("(loop M 11 seq (loop M 100 seq")     # ragged: ceil
    assert rw("(seq (mark grid) (split M 128))", NEST)[0] == b.ELEVATE_FAILED  # only sequential loops split


def test_interchange_swaps_adjacent_loops_of_different_axes():
    assert rw("interchange", NEST)[1] == "(loop N 512 seq (loop M 1024 seq (loop K 256 seq mac)))"
    assert rw("(seq interchange interchange)", NEST)[1] == NEST
    assert rw("(seq (split M 128) interchange)", NEST)[0] == b.ELEVATE_FAILED   # two halves of one split loop
    assert rw("(bodyN 2 interchange)", NEST)[0] == b.ELEVATE_FAILED             # K has no loop below it


def test_tile_is_split_split_interchange():
    tiled = "(loop M 8 seq (loop N 4 seq (loop M 128 seq (loop N 128 seq (loop K 256 seq mac)))))"
    code, out, steps, trace = b.elevate_rewrite("(tile 128 128)", NEST, trace=True)
    assert (code, out, steps) == (0, tiled, 3)
    assert [ln.split(":")[0] for ln in trace.strip().split("\n")] == ["split(M,128)", "split(N,128)", "interchange"]
    by_hand = "(seq (split M 128) (bodyN 2 (split N 128)) (body interchange))"
    assert rw(by_hand, NEST)[1] == tiled


def test_reorder_is_built_from_interchanges():
    code, out, steps = rw("(reorder 2 0 1)", NEST)
    assert (code, out) == (0, "(loop K 256 seq (loop M 1024 seq (loop N 512 seq mac)))") and steps == 2
    assert rw("(reorder 0 1 2)", NEST) == (0, NEST, 0)
    assert rw("(reorder 1 0 1)", NEST)[0] == b.ELEVATE_EPARSE
    assert rw("(reorder 0 1 2 3)", NEST)[0] == b.ELEVATE_FAILED              # only three loops
    # loops of one axis keep their order: moving the inner half of a split loop above the outer fails
    assert rw("(seq (split M 128) (reorder 1 0))", NEST)[0] == b.ELEVATE_FAILED


def test_marks_are_only_applicable_where_the_choice_is_valid():
    assert rw("(mark grid)", NEST)[1].startswith("(loop M 1024 grid")
    assert rw("(mark wave)", NEST)[1].startswith("(loop M 1024 wave")
    assert rw("(bodyN 2 (mark wave))", NEST)[0] == b.ELEVATE_FAILED          # not over the reduction
    assert rw("(mark slab)", NEST)[0] == b.ELEVATE_FAILED                    # a slab loop is a K loop
    assert rw("(bodyN 2 (mark slab))", NEST)[1].endswith("(loop K 256 slab mac)))")
    assert rw("(seq (mark grid) (mark wave))", NEST)[0] == b.ELEVATE_FAILED   # already decided
    # topDown(mark grid) twice parallelises the two outermost loops, as topDown(parallel) does in Section 6.2
    out = rw("(seq (topDown (mark grid)) (topDown (mark grid)))", NEST)[1]
    assert out == "(loop M 1024 grid (loop N 512 grid (loop K 256 seq mac)))"
    # tryAll marks every loop it can
    assert rw("(tryAll (mark unroll))", NEST)[1] == "(loop M 1024 unroll (loop N 512 unroll (loop K 256 unroll mac)))"


def test_mfma_matches_exactly_the_instruction_block():
    blk = "(loop M 32 seq (loop N 32 seq (loop K 2 seq mac)))"
    assert rw("mfma", blk) == (0, "mfma32x32x2", 1)
    assert rw("mfma", "(loop M 32 seq (loop N 32 seq (loop K 4 seq mac)))")[0] == b.ELEVATE_FAILED
    assert rw("mfma", "(loop N 32 seq (loop M 32 seq (loop K 2 seq mac)))")[0] == b.ELEVATE_FAILED
    assert rw("(topDown mfma)", f"(loop K 8 seq {blk})") == (0, "(loop K 8 seq mfma32x32x2)", 1)


def test_parse_errors():
    assert rw("(unknown x)", "x")[0] == b.ELEVATE_EPARSE
    assert rw("(seq)", "x")[0] == b.ELEVATE_EPARSE
    assert rw("(split Q 4)", "x")[0] == b.ELEVATE_EPARSE
    assert rw("(split M 0)", "x")[0] == b.ELEVATE_EPARSE
    assert rw("(mark fast)", "x")[0] == b.ELEVATE_EPARSE
    assert rw("id", "(a (b)")[0] == b.ELEVATE_EPARSE
    assert rw("id", "a b")[0] == b.ELEVATE_EPARSE
    assert rw("id", "; only a comment")[0] == b.ELEVATE_EPARSE
    assert rw("id ; trailing comment", "x") == (0, "x", 0)


# ---------------------------------------------------------------- lowering and the library's own schedules

T256 = ("(seq (tile 256 256) (bodyN 2 (tile 128 128)) (bodyN 4 (tile 32 32))"
        " (bodyN 8 (split K 16)) (bodyN 9 (split K 2))"
        " (reorder 0 1 2 3 8 9 4 5 6 7 10)"
        " (bodyN 0 (mark grid)) (bodyN 1 (mark grid)) (bodyN 2 (mark wave)) (bodyN 3 (mark wave))"
        " (bodyN 4 (mark slab)) (bodyN 6 (mark unroll)) (bodyN 7 (mark unroll)) (topDown mfma))")


def test_hand_written_schedule_of_the_large_tile_lowers_to_its_kernel():
    code, s, nest = b.elevate_schedule_gemm(4096, 4096, 4096, T256)
    assert code == 0, nest
    assert nest == ("(loop M 16 grid (loop N 16 grid (loop M 2 wave (loop N 2 wave (loop K 256 slab (loop K 8 seq "
                    "(loop M 4 unroll (loop N 4 unroll mfma32x32x2))))))))")
    assert s.as_dict() == {"bm": 256, "bn": 256, "bk": 16, "waves_m": 2, "waves_n": 2, "wave_m": 128, "wave_n": 128,
                           "split_k": 1, "tiles_m": 16, "tiles_n": 16, "k_range": 4096, "waves_k": 1}


def test_waves_sharing_the_slabs_of_one_block():
    """The 32 x 32 block whose four waves take a quarter of every 64-column slab each: K split into
    slabs, a slab into four shares of 16 columns, a share into instruction steps; `share` is valid
    for loops over K only, and only inside the staged loop."""
    text = ("(seq (bodyN 0 (split M 32)) (bodyN 3 (split K 64)) (bodyN 4 (split K 16)) (bodyN 5 (split K 2))"
            " (reorder 0 3 4 5 1 2 6)"
            " (bodyN 0 (mark grid)) (bodyN 1 (mark slab)) (bodyN 2 (mark share)) (topDown mfma))")
    code, s, nest = b.elevate_schedule_gemm(8192, 32, 8192, text)
    assert code == 0, nest
    assert nest == "(loop M 256 grid (loop K 128 slab (loop K 4 share (loop K 8 seq mfma32x32x2))))"
    assert s.as_dict() == {"bm": 32, "bn": 32, "bk": 64, "waves_m": 1, "waves_n": 1, "wave_m": 32, "wave_n": 32,
                           "split_k": 1, "tiles_m": 256, "tiles_n": 1, "k_range": 8192, "waves_k": 4}
    # the library's own choice for this shape is that kernel
    assert b.variant_name(8192, 32, 8192) == "t32x32x64k4/nn/a16"
    d = b.elevate_schedule_gemm(8192, 32, 8192, b.elevate_default_strategy(8192, 32, 8192))
    assert d[0] == 0 and d[1].as_dict() == s.as_dict()
    # not over rows or columns, not outside the staged loop
    assert b.elevate_rewrite("(mark share)", "(loop M 64 seq (loop K 8 seq mac))")[0] == b.ELEVATE_FAILED
    code, _, why = b.elevate_schedule_gemm(8192, 32, 8192, text.replace("(bodyN 1 (mark slab)) ", ""))
    assert code == b.ELEVATE_ELOWER and "outside the staged loop" in why
    # a K range that is one slab needs no staged loop: the waves share the whole range
    short = ("(seq (bodyN 2 (cover K 64)) (bodyN 0 (split M 32)) (bodyN 3 (split K 16)) (bodyN 4 (split K 2)) (reorder 0 3 4 1 2 5)"
             " (bodyN 0 (mark grid)) (bodyN 1 (mark share)) (topDown mfma))")
    code, s1, nest = b.elevate_schedule_gemm(2048, 32, 40, short)
    assert code == 0, nest
    assert nest == "(loop M 64 grid (loop K 4 share (loop K 8 seq mfma32x32x2)))"
    assert (s1.bm, s1.bn, s1.bk, s1.waves_k, s1.k_range, s1.split_k) == (32, 32, 64, 4, 64, 1)
    # but a staged loop cannot lie inside the shared one
    inside = ("(seq (bodyN 0 (split M 32)) (bodyN 3 (split K 2048)) (bodyN 4 (split K 64)) (bodyN 5 (split K 2))"
              " (reorder 0 3 4 5 1 2 6) (bodyN 0 (mark grid)) (bodyN 1 (mark share)) (bodyN 2 (mark slab)) (topDown mfma))")
    code, _, why = b.elevate_schedule_gemm(8192, 32, 8192, inside)
    assert code == b.ELEVATE_ELOWER and "inside a shared loop" in why


def test_lowering_rejects_nests_no_kernel_can_run():
    M = N = K = 4096
    # nothing scheduled: no matrix instruction
    assert b.elevate_schedule_gemm(M, N, K, "id")[0] == b.ELEVATE_ELOWER
    # grid loop inside a sequential loop
    code, _, why = b.elevate_schedule_gemm(M, N, K, T256.replace(" (bodyN 0 (mark grid))", ""))
    assert code == b.ELEVATE_ELOWER and "workgroup-parallel" in why
    # waves below a sequential loop
    code, _, why = b.elevate_schedule_gemm(M, N, K, T256.replace("(bodyN 2 (mark wave))", "(bodyN 5 (mark wave))"))
    assert code == b.ELEVATE_FAILED           # position 5 is a K loop: a wave loop over the reduction is no valid choice
    # a valid schedule whose shape no kernel has: 512 x 256 tiles
    odd = T256.replace("(tile 256 256)", "(tile 512 256)").replace("(bodyN 2 (tile 128 128))", "(bodyN 2 (tile 256 128))") \
              .replace("(bodyN 4 (tile 32 32))", "(bodyN 4 (tile 32 32))")
    code, s, nest = b.elevate_schedule_gemm(M, N, K, odd)
    assert code == b.ELEVATE_ENOKERNEL and (s.bm, s.bn, s.wave_m) == (512, 256, 256)
    # rounding M up by far more than a tile leaves workgroups with no work
    code, _, why = b.elevate_schedule_gemm(M - 1, N, K, "(seq (cover M 8192) " + T256[5:])
    assert code == b.ELEVATE_ELOWER and "no work" in why


SHAPES = [(4096, 4096, 4096), (1024, 1024, 1024), (1000, 1030, 999), (2048, 2048, 2048), (128, 128, 8192),
          (32, 32, 100000), (4095, 4097, 4099), (1, 1, 1), (64, 64, 64), (300, 70, 5), (1536, 1536, 1536),
          (384, 384, 16384), (100, 5000, 33), (8192, 32, 8192), (16, 4096, 4096), (5000, 7, 300)]


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_default_strategy_reproduces_the_dispatch_choice(M, N, K):
    """The library's own choice of tile and K split, written as a strategy, applied to the plain nest
    and lowered, gives back exactly that choice (as the dispatch reports it in its variant name)."""
    text = b.elevate_default_strategy(M, N, K)
    code, s, nest = b.elevate_schedule_gemm(M, N, K, text)
    assert code == 0, (text, nest)
    name = b.variant_name(M, N, K)
    assert name.startswith(f"t{s.bm}x{s.bn}x{s.bk}" + (f"k{s.waves_k}/" if s.waves_k > 1 else "/")), (name, s.as_dict())
    if "splitk" in name:
        assert s.split_k == int(name.split("splitk")[1])
    else:
        assert s.split_k == 1
    assert s.tiles_m == -(-M // s.bm) and s.tiles_n == -(-N // s.bn)
    grid = {(128, 32): (4, 1, 1), (32, 128): (1, 4, 1), (32, 32): (1, 1, 4), (64, 32): (1, 1, 4),
            (32, 64): (1, 1, 4)}.get((s.bm, s.bn), (2, 2, 1))                                                # waves per workgroup
    assert (s.waves_m, s.waves_n, s.waves_k, s.wave_m, s.wave_n) == (*grid, s.bm // grid[0], s.bn // grid[1])
    assert s.k_range % s.bk == 0 and s.split_k * s.k_range >= K > (s.split_k - 1) * s.k_range
    # same text, same result
    assert b.elevate_default_strategy(M, N, K) == text
    assert b.elevate_schedule_gemm(M, N, K, text)[2] == nest


def test_scheduled_entry_point_validates_on_the_host():
    lib = b.lib()
    code, s, _ = b.elevate_schedule_gemm(4096, 4096, 4096, T256)
    assert code == 0
    import ctypes
    ref = ctypes.byref(s)
    assert lib.gemm_f32_scheduled(None, 8, 8, 8, None, 8, None, 8, None, 8, 0) == -2
    assert lib.gemm_f32_scheduled(ref, 1024, 4096, 4096, None, 4096, None, 4096, None, 4096, 0) == -1   # other problem
    bad = b.Schedule.from_buffer_copy(s)
    bad.bm = 512
    assert lib.gemm_f32_scheduled(ctypes.byref(bad), 4096, 4096, 4096, None, 4096, None, 4096, None, 4096, 0) == -1
    assert lib.gemm_f32_scheduled(ref, 4096, 4096, 4096, None, 4096, None, 4096, None, 4096, 0) == -2      # null operands


# ---------------------------------------------------------------- Section 5: the binomial filter

BF = ("(fun img (map2D (fun nbh (reduce add 0 (map mult (zip (join weights2d) (join nbh))))) "
      "(slide2D 3 1 (pad2D 1 img))))")
SEPARATE = "(topDown (separateDot weights2d weightsH weightsV))"


def test_separate_dot_rewrites_the_naive_filter_as_section_5_2_prints_it():
    code, out, steps = rw(SEPARATE, BF)
    # nbh |> map(dot(weightsH)) |> dot(weightsV), inside the unchanged pad / slide / map2D pipeline
    assert (code, steps) == (0, 1)
    assert out == ("(fun img (map2D (fun nbh (dot weightsV (map (dot weightsH) nbh))) "
                   "(slide2D 3 1 (pad2D 1 img))))")
    # the underlined parts of the pattern must match: other weights, another operator, no match
    assert rw("(topDown (separateDot otherWeights weightsH weightsV))", BF)[0] == b.ELEVATE_FAILED
    assert rw(SEPARATE, BF.replace("add", "max"))[0] == b.ELEVATE_FAILED
    assert rw(SEPARATE, BF.replace("mult", "add"))[0] == b.ELEVATE_FAILED
    assert rw(SEPARATE, out)[0] == b.ELEVATE_FAILED                     # already separated
    assert rw("(separateDot weights2d weightsH weightsV)", BF)[0] == b.ELEVATE_FAILED   # not at the root


def test_filter_strategies_select_the_three_kernels():
    assert b.elevate_schedule_filter("id")[:2] == (0, 0)                                 # naive
    code, form, prog = b.elevate_schedule_filter(f"(seq {SEPARATE} (topDown (storeRows image)))")
    assert (code, form) == (0, 1) and "(stored image (map (dot weightsH) nbh))" in prog   # separated
    code, form, prog = b.elevate_schedule_filter(f"(seq {SEPARATE} (topDown (storeRows line)))")
    assert (code, form) == (0, 2) and "(stored line " in prog                             # scanline
    # separated but nobody said where the row sums live: no kernel
    code, form, why = b.elevate_schedule_filter(SEPARATE)
    assert code == b.ELEVATE_ELOWER and form == -1 and "stored" in why
    # the storage choice is only valid on the separated form
    assert b.elevate_schedule_filter("(topDown (storeRows line))")[0] == b.ELEVATE_FAILED
    twice = f"(seq {SEPARATE} (topDown (storeRows line)) (topDown (storeRows image)))"
    assert b.elevate_schedule_filter(twice)[0] == b.ELEVATE_FAILED
    assert b.elevate_schedule_filter("(storeRows nowhere)")[0] == b.ELEVATE_EPARSE


# ---------------------------------------------------------------- Section 6.1: the tutorial's loop orders

def test_blocking_and_loop_permutation_schedules_give_the_loop_orders_of_section_6_1():
    """blocking: tile(32,32) on the two outer loops, split k by 4, reorder (xo, yo, ko, ki, xi, yi);
    loop permutation: the same with ki and xi switched: (xo, yo, ko, xi, ki, yi)."""
    nest = "(loop M 1024 seq (loop N 1024 seq (loop K 1024 seq mac)))"

    def order(text):
        import re
        return re.findall(r"[(]loop ([MNK]) ([0-9]+)", text)

    blocking = "(seq (tile 32 32) (bodyN 4 (split K 4)) (reorder 0 1 4 5 2 3))"
    code, out, _ = rw(blocking, nest)
    assert code == 0
    assert order(out) == [("M", "32"), ("N", "32"), ("K", "256"), ("K", "4"), ("M", "32"), ("N", "32")]
    permuted = "(seq (tile 32 32) (bodyN 4 (split K 4)) (reorder 0 1 4 2 5 3))"
    code, out, _ = rw(permuted, nest)
    assert code == 0
    assert order(out) == [("M", "32"), ("N", "32"), ("K", "256"), ("M", "32"), ("K", "4"), ("N", "32")]
    # from the blocking order, switching ki and xi is one interchange at depth 3
    assert rw(f"(seq {blocking} (bodyN 3 interchange))", nest)[1] == out
    # parallelising the outermost loop (the tutorial's last version) is topDown(mark grid)
    assert rw(f"(seq {permuted} (topDown (mark grid)))", nest)[1].startswith("(loop M 32 grid (loop N 32 seq")


def test_dispatch_plans_from_the_lowered_nest_on_the_survey_shapes():
    """The production dispatch realises every choice through the strategy layer: for the 92 shapes of the
    benchmark's survey (52 fixed, 40 seeded random, either layout of B) the plan is built from the configuration
    lowered from the nest that (lChoice (seq admissible cheapest schedule) ...) rewrote, never from the cost
    model's answer as it stood; and where the layer can be asked from outside (B stored K x N), the strategy
    text it prints lowers to the tile and split of the plan."""
    import importlib.util
    import math
    import os
    import random
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location("bench_module_for_elevate", os.path.join(root, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    rng = random.Random(3)
    shapes = list(bench.SURVEY_SHAPES)
    while len(shapes) < len(bench.SURVEY_SHAPES) + 40:
        M, N, K = (int(round(math.exp(rng.uniform(math.log(a), math.log(b))))) for a, b in ((32, 4096), (32, 4096), (64, 8192)))
        if 2.0 * M * N * K <= 4e10:
            shapes.append((M, N, K, rng.random() < 0.5))
    assert len(shapes) == 92
    b.set_test_hooks()
    applied0, failed0 = b.elevate_dispatch_stats()
    # shapes nobody has asked about yet in this process: shifted by a prime so that the process-wide table misses
    fresh = [(M + 7, N, K, tB) for (M, N, K, tB) in shapes]
    names = [b.variant_name(M, N, K, transB=tB) for (M, N, K, tB) in shapes + fresh]
    applied1, failed1 = b.elevate_dispatch_stats()
    assert failed1 == failed0 == 0
    assert applied1 - applied0 >= len(set(fresh))
    for (M, N, K, tB), name in zip(shapes + fresh, names):
        if tB or name.startswith("thin"):
            continue
        rc, sched, _ = b.elevate_schedule_gemm(M, N, K, b.elevate_default_strategy(M, N, K))
        assert rc == 0, (M, N, K)
        parts = name.split("/")
        tile = f"t{sched.bm}x{sched.bn}x{sched.bk}" + (f"k{sched.waves_k}" if sched.waves_k > 1 else "")
        assert parts[0] == tile, (M, N, K, name, sched.as_dict())
        split = [int(x[len("splitk"):]) for x in parts if x.startswith("splitk")]
        assert sched.split_k == (split[0] if split else 1), (M, N, K, name, sched.as_dict())
