"""Host logic behind the GEMM entry points, without a GPU: which kernel a shape takes, how the large-M kernel cuts it
into whole and half tiles, how many workgroups share a tile along K, and what the workspace must hold -- checked as
properties over a grid of shapes on a 256-compute-unit device (fq_w4a8_gemm_plan launches nothing)."""
import itertools

from paper_2505_20839_amd import binding

CUS = 256
MS = [1, 16, 17, 56, 57, 64, 65, 100, 128, 129, 192, 256, 300, 384, 512, 513, 1024, 2048, 8192]
NS = [32, 64, 96, 200, 512, 1000, 4096, 6144, 8192, 11008, 14336, 16384, 16448, 22016, 28672]
KS = [128, 256, 1024, 1408, 4096, 5120, 8192, 11008, 16384]


def _plan(M, N, K):
    return binding.fq_w4a8_gemm_plan(M, N, K, CUS)


def test_kernel_choice_follows_m_and_the_tile_count():
    binding.fq_test_force_kernel(None)
    for M, N, K in itertools.product(MS, NS, KS):
        p = _plan(M, N, K)
        if M <= 16:
            assert p["kernel"] == "small16", (M, N, K)
        elif M <= 64:
            tiles64 = -(-N // 64)
            top = M > 56 and 8 <= K // 128 <= 64 and tiles64 <= CUS <= 2 * tiles64
            assert p["kernel"] == ("ksplit64x64" if top else "smallm"), (M, N, K)
            if top:
                assert p["ksplit_tiles"] == tiles64 and p["ksplit_slices"] == 1
        else:
            tiles = -(-M // 128) * -(-N // 64)
            rounds = 2 if (M <= 128 and K // 128 >= 40) else 1
            want_ksplit = M <= 512 and K // 128 >= 8 and tiles <= rounds * CUS
            assert (p["kernel"] == "ksplit128x64") == want_ksplit, (M, N, K, p)
            if not want_ksplit:
                assert p["kernel"] == "large", (M, N, K, p)


def test_large_kernel_tiles_cover_the_problem_once():
    """Whole tiles count 256 rows, half tiles 128: together they cover every 128-row x 128-channel block of the
    padded problem exactly once."""
    binding.fq_test_force_kernel("large")
    try:
        for M, N, K in itertools.product([65, 128, 300, 513, 2048, 2100, 8192], NS, [256, 4096]):
            p = _plan(M, N, K)
            assert p["kernel"] == "large"
            tiles_n = -(-N // 128)
            whole, half = p["whole"] + p["whole_ragged"], p["half"] + p["half_ragged"]
            tiles_m = -(-M // 256)
            # a whole tile whose second half lies past M still counts two blocks of the padded problem; halves that
            # start past M are not launched
            blocks = 2 * whole + half
            lo = -(-M // 128) * tiles_n                       # every block that holds a row must be covered
            hi = 2 * tiles_m * tiles_n
            assert lo <= blocks <= hi, (M, N, K, p)
            if M % 256 == 0 and N % 128 == 0 and N % 8 == 0:
                assert p["whole_ragged"] == 0 and p["half_ragged"] == 0 and blocks == hi
    finally:
        binding.fq_test_force_kernel(None)


def test_k_slices_fill_the_device_without_empty_slices():
    binding.fq_test_force_kernel(None)
    seen_sliced = 0
    for M, N, K in itertools.product(MS, NS, KS):
        p = _plan(M, N, K)
        if p["kernel"] != "ksplit128x64":
            assert p["ksplit_slices"] == 0 or p["kernel"].startswith("ksplit")
            continue
        S, G = p["ksplit_slices"], K // 128
        tiles = p["ksplit_tiles"]
        assert tiles == -(-M // 128) * -(-N // 64)
        assert 1 <= S <= 8
        if S > 1:
            seen_sliced += 1
            assert tiles * S <= CUS                            # one round of the compute units
            assert G // S >= 8 or -(-G // S) >= 8              # two groups or more for each of a workgroup's four K splits
            per = -(-G // S)
            assert per * (S - 1) < G                           # the last slice is not empty
        else:
            # no further slice would fit, or K is too short to share
            assert tiles * 2 > CUS or G // 8 < 2 or (-(-G // 2)) * 1 >= G
    assert seen_sliced > 50


def test_workspace_holds_planes_counters_and_partial_tiles():
    binding.fq_test_force_kernel(None)
    for M, N, K in itertools.product(MS, NS, KS):
        p = _plan(M, N, K)
        need = binding.fq_w4a8_gemm_workspace_bytes(M, N, K)
        if M <= 64:
            assert need == 0
            continue
        G = K // 128
        planes = 2 * (2 * -(-G // 16)) * M * 16
        counters = 4096 if M <= 512 else 0
        partial = 0
        if p["kernel"] == "ksplit128x64" and p["ksplit_slices"] > 1:
            partial = p["ksplit_slices"] * p["ksplit_tiles"] * 128 * 64 * 4
        assert need == planes + counters + partial, (M, N, K, p, need)
        assert partial <= 8 << 20                              # what the built-in scratch of the static entry point allows for
