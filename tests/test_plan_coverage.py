"""CPU-only: the layer-step parity cases together reach every GEMM kernel variant the library can pick.

faar_gemm_plan is a pure host function that reports the variant (tile shape, slice width, contraction split)
the library uses for each GEMM of a layer.  The set of (GEMM, variant, split or not) combinations that ANY layer
shape can produce is found by scanning a wide grid of shapes; the parity cases must cover all of it, so that no
kernel instantiation runs in the benchmark without having been compared with the oracle."""
import itertools

from paper_2603_22370_amd import binding as fb

from parity_cases import GRAM_CASES, STEP_CASES

GEMMS = {"residual": fb.K_GEMM_RESIDUAL, "dw": fb.K_GEMM_DW, "dx": fb.K_GEMM_DX, "c": fb.K_GEMM_C}
DIMS = [16, 32, 48, 64, 80, 96, 128, 160, 192, 224, 256, 288, 320, 384, 448, 512, 640, 768, 1024, 1280, 1536, 2048,
        2560, 3072, 4096, 6144, 8192, 12288, 14336, 16384]
TOKENS = [1, 3, 33, 64, 65, 100, 128, 256, 300, 512, 640, 1024, 1536, 2048, 3072, 4096, 8192, 16384, 65536]


# shapes (O, K, T) on which tests/test_gpu_block.py compares faar_linear_forward with the oracle
FORWARD_CASES = [(96, 80, 100), (640, 256, 300), (2048, 512, 1024), (6144, 2048, 2048), (640, 256, 300), (256, 640, 300)]


def _combos(O, K, T, chained):
    for g, which in GEMMS.items():
        if g == "dx" and not chained:
            continue
        kind, bm, bn, split = fb.faar_gemm_plan(which, O, K, T)
        yield (g, kind, (bm, bn), "split" if split > 1 else "whole")


def test_parity_cases_reach_every_gemm_variant():
    reachable = {}
    for O, K, T in itertools.product(DIMS, DIMS, TOKENS):
        if O * K * T > 2 ** 40:
            continue
        for combo in _combos(O, K, T, chained=(O % 8 == 0)):
            reachable.setdefault(combo, (O, K, T))
    covered = set()
    for c in STEP_CASES:
        covered.update(_combos(c.O, c.K, c.T, c.chained))
    missing = {k: v for k, v in reachable.items() if k not in covered}
    assert not missing, f"variants no parity case reaches (with an example shape): {missing}"
    # every variant name the library knows is reachable by some GEMM, so none is dead code
    assert {k[1] for k in reachable} == set(fb.GEMM_KINDS)


def test_benchmark_shapes_are_parity_cases_at_full_size():
    """Every (variant, split) the Llama3-1B- and Qwen3-1.7B-shaped linears take at the benchmark's token counts is
    also taken by a full-size parity case (several contraction slices, ring wrap-around, all tiles)."""
    llama = [(2048, 2048), (512, 2048), (8192, 2048), (2048, 8192)]
    qwen = [(2048, 2048), (1024, 2048), (6144, 2048), (2048, 6144)]
    full = set()
    for c in STEP_CASES:
        if c.full_size:
            full.update(_combos(c.O, c.K, c.T, c.chained))
    for shapes, T, chained in ((llama, 4096, False), (qwen, 8192, False), (qwen, 16384, True)):
        for O, K in shapes:
            for combo in _combos(O, K, T, chained):
                if combo[1] in ("L64", "M64"):          # the two fast kernels; the 128x128 one is covered by small cases
                    assert combo in full, (O, K, T, combo)


def test_forward_gemm_of_the_joint_step_runs_kernels_that_parity_cases_cover():
    """faar_linear_forward uses the bf16-output GEMM (the dX GEMM's epilogue) on T x O x K: every variant it takes on the
    joint benchmark's shapes is a variant some parity case reaches with that epilogue (as dX GEMM or as forward GEMM)."""
    covered = set()
    for c in STEP_CASES:
        if c.chained:
            kind, bm, bn, _ = fb.faar_gemm_plan(fb.K_GEMM_DX, c.O, c.K, c.T)
            covered.add((kind, bm, bn))
    for O, K, T in FORWARD_CASES:
        kind, bm, bn, _ = fb.faar_gemm_plan(fb.K_GEMM_FWD, O, K, T)
        covered.add((kind, bm, bn))
    for O, K in ((6144, 2048), (2048, 6144)):
        kind, bm, bn, _ = fb.faar_gemm_plan(fb.K_GEMM_FWD, O, K, 16384)
        assert (kind, bm, bn) in covered, (O, K, kind)


def test_gram_form_product_runs_kernels_that_its_parity_cases_cover():
    """The O x K x K product of faar_layer_step_gram: every (variant, tile, split or not) any layer shape can take is taken
    by one of the cases tests/test_gpu_gram.py runs (all of STEP_CASES and GRAM_CASES), and the benchmark's layer shapes by full-size ones."""
    def combo(O, K):
        kind, bm, bn, split = fb.faar_gemm_plan(fb.K_GEMM_GRAM, O, K, 1)
        return (kind, (bm, bn), "split" if split > 1 else "whole")

    reachable = {}
    for O, K in itertools.product(DIMS, DIMS):
        if K % 16 == 0:
            reachable.setdefault(combo(O, K), (O, K))
    covered = {combo(c.O, c.K) for c in STEP_CASES + GRAM_CASES}
    missing = {k: v for k, v in reachable.items() if k not in covered}
    assert not missing, f"Gram-form variants no parity case reaches (with an example shape): {missing}"
    full = {combo(c.O, c.K) for c in STEP_CASES if c.full_size}
    for O, K in [(2048, 2048), (512, 2048), (8192, 2048), (2048, 8192), (1024, 2048), (6144, 2048), (2048, 6144)]:
        assert combo(O, K) in full, (O, K, combo(O, K))


def test_token_major_residual_gemm_runs_kernels_that_parity_cases_cover():
    """Where faar_dw_token_major holds, a step that carries the constant as H leaves dY token-major: its residual GEMM is the
    T x O x K product planned like the forward GEMM, with an epilogue of its own.  Every variant that product can take on such
    a shape is taken by a parity case (each runs once with H, no upstream gradient and no dX), and the benchmark's by
    full-size ones."""
    def combo(O, K, T):
        kind, bm, bn, _ = fb.faar_gemm_plan(fb.K_GEMM_FWD, O, K, T)
        return (kind, (bm, bn))

    reachable = {}
    for O, K, T in itertools.product(DIMS, DIMS, TOKENS):
        if O * K * T <= 2 ** 40 and fb.faar_dw_token_major(O, K, T):
            reachable.setdefault(combo(O, K, T), (O, K, T))
    covered = {combo(c.O, c.K, c.T) for c in STEP_CASES if fb.faar_dw_token_major(c.O, c.K, c.T)}
    missing = {k: v for k, v in reachable.items() if k not in covered}
    assert not missing, f"token-major residual variants no parity case reaches (with an example shape): {missing}"
    full = {combo(c.O, c.K, c.T) for c in STEP_CASES if c.full_size and fb.faar_dw_token_major(c.O, c.K, c.T)}
    for O, K in [(2048, 2048), (1024, 2048), (6144, 2048), (2048, 6144)]:
        assert not fb.faar_dw_token_major(O, K, 8192) or combo(O, K, 8192) in full, (O, K)
    assert fb.faar_dw_token_major(6144, 2048, 8192) and fb.faar_dw_token_major(2048, 6144, 8192)


def test_token_major_dw_gemm_tiles_are_all_reached_by_parity_cases():
    """The token-major dW GEMM has three tile shapes (two of them only for a step that has the device to itself), each whole or
    with the contraction split: every combination some layer shape takes is taken by a parity case (each runs it with H and
    its own gradient; chained ones also with an upstream one)."""
    def combo(O, K, T, whole_device):
        return (fb.faar_dw_token_major(O, K, T, whole_device), "split" if fb.faar_gemm_plan(fb.K_GEMM_DW, O, K, T)[3] > 1 else "whole")

    reachable = {}
    dims = DIMS + [528, 1032, 1312, 6576, 7248, 8088]
    for O, K, T in itertools.product(dims, dims, TOKENS):
        if O * K * T <= 2 ** 40 and fb.faar_dw_token_major(O, K, T):
            assert fb.faar_dw_token_major(O, K, T) == 1
            for whole_device in (False, True):
                reachable.setdefault(combo(O, K, T, whole_device), (O, K, T))
    assert {k[0] for k in reachable} == {1, 2, 3}
    token_major = [c for c in STEP_CASES if fb.faar_dw_token_major(c.O, c.K, c.T)]
    covered = {combo(c.O, c.K, c.T, c.whole_device) for c in token_major}
    missing = {k: v for k, v in reachable.items() if k not in covered}
    assert not missing, f"token-major dW variants no parity case reaches (with an example shape): {missing}"
    assert {combo(c.O, c.K, c.T, c.whole_device)[0] for c in token_major if c.chained} == {1, 2, 3}
    # alone on the device, the default benchmark's two large shapes take the 192-wide tiles, and full-size parity cases run them
    full = {combo(c.O, c.K, c.T, c.whole_device) for c in STEP_CASES if c.full_size}
    assert combo(6144, 2048, 8192, True) == (2, "whole") and combo(2048, 6144, 8192, True) == (3, "whole")
    assert combo(6144, 2048, 8192, True) in full and combo(2048, 6144, 8192, True) in full
    # ... and beside other streams 256 x 256 ones, split or not, which full-size cases run as well
    assert {(1, "whole"), (1, "split")} <= full
