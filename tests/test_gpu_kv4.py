"""GPU parity of the attention operands with an INT4 key/value cache (fq_kv4_*) against the CPU oracle:
cache packing bit-exact, scores and outputs element by element within one bf16 step + 1e-3 of the sum of |terms|."""
import numpy as np
import pytest

import oracle
from paper_2505_20839_amd import workloads
from parity_util import bf16_bits_from_gpu, check_gemm, to_gpu_bf16

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def fq():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: torch.cuda.is_available() is False")
    from paper_2505_20839_amd import binding
    binding.lib()
    return binding


def _gpu(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _codes(rng, shape, top=0x78, signed=True):
    c = rng.integers(0, top, shape).astype(np.uint8)
    return c | (rng.integers(0, 2, shape).astype(np.uint8) << 7) if signed else c


@pytest.mark.parametrize("H,T", [(1, 1), (3, 32), (2, 100), (5, 129), (8, 4096), (2, 1000)])
def test_cache_pack_roundtrip(fq, H, T):
    rng = np.random.default_rng(H + T)
    codes = rng.integers(-8, 8, (H, T, 128), dtype=np.int8)
    for values in (False, True):
        packed = fq.fq_kv4_pack(_gpu(codes), values)
        assert packed.numel() == fq.lib().fq_kv4_packed_bytes(H, T, int(values))
        assert np.array_equal(fq.fq_kv4_unpack(packed, H, T, values).cpu().numpy(), codes)
    # a key cache is the linear-layer packing of each head's [T, 128] matrix
    kp = fq.fq_kv4_pack(_gpu(codes), False).cpu().numpy().reshape(H, -1)
    for h in range(min(H, 2)):
        assert np.array_equal(kp[h], fq.fq_pack_weights(_gpu(codes[h])).cpu().numpy())


SCORE_SHAPES = [(1, 1, 1), (2, 4, 100), (3, 16, 256), (2, 17, 300), (1, 64, 513), (8, 4, 4096), (5, 33, 70), (2, 64, 516),
                (3, 5, 4)]


@pytest.mark.parametrize("H,R,T", SCORE_SHAPES)
def test_scores_match_the_oracle(fq, H, R, T):
    rng = np.random.default_rng(H * 1000 + R * 10 + T)
    Q = _codes(rng, (H, R, 128)); Kq = rng.integers(-8, 8, (H, T, 128), dtype=np.int8)
    ks = _codes(rng, (H, T), top=0x50); qs = rng.uniform(0.01, 2, (H, R)).astype(np.float32)
    ks[:, T // 2] = 0                                          # a token with scale zero scores zero
    S = fq.fq_kv4_scores(_gpu(Q), _gpu(qs), fq.fq_kv4_pack(_gpu(Kq), False), _gpu(ks), 0.088388346)
    torch.cuda.synchronize()
    Sr, B = oracle.kv4_scores(Q, qs, Kq, ks, 0.088388346, want_bound=True)
    got = bf16_bits_from_gpu(S)
    # (the norm-wise criterion needs enough outputs for the bf16 rounding errors to average out)
    check_gemm(got.reshape(H * R, T), Sr.reshape(H * R, T), B.reshape(H * R, T), "scores %s" % ((H, R, T),),
               frobenius=H * R * T >= 20000)
    assert not oracle.bf16_bits_to_f64(got)[:, :, T // 2].any()


# (T a multiple of 16 with the padded stride below: the kernel of 16-byte steps; 144 and 1040 end inside a 128-token group)
OUTPUT_SHAPES = [(1, 1, 1), (2, 4, 100), (3, 16, 256), (2, 17, 300), (1, 32, 513), (8, 4, 4096), (5, 9, 70), (2, 20, 144),
                 (3, 4, 1040), (1, 1, 16), (40, 16, 272),
                 # heads enough for 2 and for 4 dimension tiles per workgroup on a 256-unit device (1 below 64 heads)
                 (70, 4, 144), (130, 3, 272), (260, 20, 48)]


@pytest.mark.parametrize("H,R,T", OUTPUT_SHAPES)
def test_outputs_match_the_oracle(fq, H, R, T):
    rng = np.random.default_rng(H * 1000 + R * 10 + T + 7)
    ldp = T + (-T) % 16 + 16                                   # a padded row stride; the padding holds junk that must not be read as data
    P = _codes(rng, (H, R, ldp), top=0x7F, signed=False)
    Vq = rng.integers(-8, 8, (H, T, 128), dtype=np.int8)
    vs = _codes(rng, (H, T), top=0x50); ps = rng.uniform(0.001, 0.1, (H, R)).astype(np.float32)
    vs[:, 0] = 0x7E                                            # the largest scale next to the largest probabilities
    O = fq.fq_kv4_output(_gpu(P), _gpu(ps), fq.fq_kv4_pack(_gpu(Vq), True), _gpu(vs))
    torch.cuda.synchronize()
    Or, B = oracle.kv4_output(P[:, :, :T], ps, Vq, vs, want_bound=True)
    check_gemm(bf16_bits_from_gpu(O).reshape(H * R, 128), Or.reshape(H * R, 128), B.reshape(H * R, 128),
               "output %s" % ((H, R, T),), frobenius=False)   # (token 0 carries the largest scale and most of the norm)


def test_one_hot_operands_read_back_every_cache_element(fq):
    """A one-hot query reads one key element per token, a one-hot probability row one token's values: every packed
    code and every scale of both caches arrives where the oracle says (exact products: only bf16 rounding left)."""
    H, T = 2, 160
    rng = np.random.default_rng(3)
    Kq = rng.integers(-8, 8, (H, T, 128), dtype=np.int8); Vq = rng.integers(-8, 8, (H, T, 128), dtype=np.int8)
    ks = rng.integers(1, 0x50, (H, T)).astype(np.uint8); vs = rng.integers(1, 0x50, (H, T)).astype(np.uint8)
    kp, vp = fq.fq_kv4_pack(_gpu(Kq), False), fq.fq_kv4_pack(_gpu(Vq), True)
    for r0 in range(0, 128, 64):
        Q = np.zeros((H, 64, 128), np.uint8); Q[:, np.arange(64), r0 + np.arange(64)] = 0x38
        one = np.ones((H, 64), np.float32)
        S = bf16_bits_from_gpu(fq.fq_kv4_scores(_gpu(Q), _gpu(one), kp, _gpu(ks), 1.0))
        want = oracle.kv4_scores(Q, one, Kq, ks, 1.0)
        assert np.array_equal(oracle.bf16_bits_to_f64(S), oracle.bf16_bits_to_f64(oracle.bf16_round_array(want)))
    for t0 in range(0, T, 32):
        P = np.zeros((H, 32, T), np.uint8); P[:, np.arange(32), t0 + np.arange(32)] = 0x38
        one = np.ones((H, 32), np.float32)
        O = bf16_bits_from_gpu(fq.fq_kv4_output(_gpu(P), _gpu(one), vp, _gpu(vs)))
        want = oracle.kv4_output(P, one, Vq, vs)
        assert np.array_equal(oracle.bf16_bits_to_f64(O), oracle.bf16_bits_to_f64(oracle.bf16_round_array(want)))


def test_decode_attention_operands_on_a_cache_of_workload_size(fq):
    """Llama3-8B decode: 8 key/value heads x a batch of 4 sequences, 4 query heads each, 4096 cached tokens; queries
    and probabilities quantised by fq_quantize_act as everywhere else in the path."""
    H, R, T = 32, 4, 4096
    d = workloads.draw_kv_cache(H, R, T, seed=11)
    Qc, qs = fq.fq_quantize_act(to_gpu_bf16(d["Q_bf16"].reshape(H * R, 128)))
    Pc, ps = fq.fq_quantize_act(to_gpu_bf16(d["P_bf16"].reshape(H * R, T)))
    kp, vp = fq.fq_kv4_pack(_gpu(d["Kq"]), False), fq.fq_kv4_pack(_gpu(d["Vq"]), True)
    S = fq.fq_kv4_scores(Qc.view(H, R, 128), qs.view(H, R), kp, _gpu(d["k_scale"]), 128 ** -0.5)
    O = fq.fq_kv4_output(Pc.view(H, R, T), ps.view(H, R), vp, _gpu(d["v_scale"]))
    torch.cuda.synchronize()
    Qn, qn = Qc.cpu().numpy().reshape(H, R, 128), qs.cpu().numpy().reshape(H, R)
    Pn, pn = Pc.cpu().numpy().reshape(H, R, T), ps.cpu().numpy().reshape(H, R)
    Sr, SB = oracle.kv4_scores(Qn, qn, d["Kq"], d["k_scale"], 128 ** -0.5, want_bound=True)
    Or, OB = oracle.kv4_output(Pn, pn, d["Vq"], d["v_scale"], want_bound=True)
    check_gemm(bf16_bits_from_gpu(S).reshape(H * R, T), Sr.reshape(H * R, T), SB.reshape(H * R, T), "decode scores")
    check_gemm(bf16_bits_from_gpu(O).reshape(H * R, 128), Or.reshape(H * R, 128), OB.reshape(H * R, 128), "decode output")
