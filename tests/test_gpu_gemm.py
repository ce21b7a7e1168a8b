"""GPU parity of the contraction primitive in all three operand layouts, against fp64 matmul
on the same bf16-rounded inputs: ragged M / K, several terms, accumulate."""
import numpy as np
import pytest
import torch

import synth_inputs as synth
from helpers import to_dev, to_np, rel_err

pytestmark = pytest.mark.gpu


def operands(rng, M, N, K, a_k, b_k, dtype):
    A = synth.quantize(rng.standard_normal((M, K) if a_k else (K, M)).astype(np.float32), dtype)
    B = synth.quantize(rng.standard_normal((N, K) if b_k else (K, N)).astype(np.float32), dtype)
    A64 = A.astype(np.float64) if a_k else A.astype(np.float64).T
    B64 = B.astype(np.float64).T if b_k else B.astype(np.float64)
    return A, B, A64 @ B64


@pytest.mark.parametrize("a_k,b_k", [(True, False), (False, False), (True, True)])
@pytest.mark.parametrize("M,N,K", [(256, 256, 64), (700, 512, 192), (1000, 768, 333 * 8), (37, 256, 128)])
def test_gemm_layouts_bf16(a_k, b_k, M, N, K):
    import paper_2503_01066_amd as A_
    if (a_k or b_k) and K % 64:
        K = (K // 64) * 64
    if not a_k:
        M = (M + 7) // 8 * 8
    rng = np.random.default_rng(M * 7 + N + K)
    A, B, ref = operands(rng, M, N, K, a_k, b_k, "bf16")
    C = A_.alch_gemm(M, N, [(to_dev(A, "bf16"), to_dev(B, "bf16"), K)], a_k, b_k)
    torch.cuda.synchronize()
    assert rel_err(to_np(C), ref) < 6e-3       # one bf16 rounding of the output


def test_gemm_terms_accumulate_and_fp32():
    import paper_2503_01066_amd as A_
    rng = np.random.default_rng(0)
    M, N = 300, 512
    A1, B1, r1 = operands(rng, M, N, 128, True, False, "bf16")
    A2, B2, r2 = operands(rng, M, N, 192, True, False, "bf16")
    C0 = synth.quantize(rng.standard_normal((M, N)).astype(np.float32) * 10, "bf16")
    C = to_dev(C0, "bf16")
    A_.alch_gemm(M, N, [(to_dev(A1, "bf16"), to_dev(B1, "bf16"), 128), (to_dev(A2, "bf16"), to_dev(B2, "bf16"), 192)],
                 True, False, out=C, accumulate=True)
    torch.cuda.synchronize()
    assert rel_err(to_np(C), r1 + r2 + C0) < 6e-3
    A3, B3, r3 = operands(rng, 70, 45, 33, False, False, "f32")
    C = A_.alch_gemm(70, 45, [(to_dev(A3, "f32"), to_dev(B3, "f32"), 33)], False, False)
    torch.cuda.synchronize()
    assert rel_err(to_np(C), r3) < 1e-5


@pytest.mark.parametrize("a_k,b_k", [(False, False), (True, False), (True, True)])
@pytest.mark.parametrize("M,N,K,acc", [(6144, 4096, 2048, False),     # 384 tiles: last round of 128, two parts each
                                       (2040, 10232, 4096, True),     # 320 tiles with ragged edges: last round of 64, four parts
                                       (2048, 10240, 1024, False)])   # contraction too short for four parts: not split
def test_gemm_split_last_round(a_k, b_k, M, N, K, acc):
    # with scratch the tiles of a half-empty last round are split along K; the result is that of the plain launch
    # up to fp32 summation order, and both agree with fp64
    import paper_2503_01066_amd as A_
    rng = np.random.default_rng(M + N + K)
    A, B, ref = operands(rng, M, N, K, a_k, b_k, "bf16")
    C0 = synth.quantize(rng.standard_normal((M, N)).astype(np.float32) * 30, "bf16")
    dA, dB = to_dev(A, "bf16"), to_dev(B, "bf16")
    ws = torch.empty(A_.lib().alch_gemm_workspace_bytes(), dtype=torch.uint8, device="cuda")
    outs = []
    for w in (None, ws, ws):
        C = to_dev(C0, "bf16")
        A_.alch_gemm(M, N, [(dA, dB, K)], a_k, b_k, out=C, accumulate=acc, workspace=w)
        torch.cuda.synchronize()
        outs.append(to_np(C))
    want = ref + C0 if acc else ref
    assert rel_err(outs[0], want) < 6e-3
    assert rel_err(outs[1], want) < 6e-3
    assert np.array_equal(outs[1], outs[2])                      # deterministic
    assert rel_err(outs[1], outs[0]) < 1e-2                      # at most a last-bit difference of the rounded output


@pytest.mark.parametrize("a_k,b_k,M,N,Ks", [(True, False, 256, 4096, (4096, 2048)),      # 16 tiles, two operand pairs, 12 parts
                                            (True, False, 300, 4096, (1024, 512, 6144)),  # ragged rows, parts crossing pair boundaries
                                            (True, True, 512, 1024, (8192,)),              # 8 tiles, 16 parts
                                            (False, False, 2048, 1024, (2048,))])          # 32 tiles, 4 parts
def test_gemm_split_short_batches(a_k, b_k, M, N, Ks):
    # a product with tiles for at most half of the compute units splits every tile along the contraction,
    # across the operand pairs in order
    import paper_2503_01066_amd as A_
    rng = np.random.default_rng(M + N + sum(Ks))
    terms, ref = [], 0.0
    for K in Ks:
        A, B, r = operands(rng, M, N, K, a_k, b_k, "bf16")
        terms.append((to_dev(A, "bf16"), to_dev(B, "bf16"), K))
        ref = ref + r
    ws = torch.empty(A_.lib().alch_gemm_workspace_bytes(), dtype=torch.uint8, device="cuda")
    C0 = A_.alch_gemm(M, N, terms, a_k, b_k)
    C1 = A_.alch_gemm(M, N, terms, a_k, b_k, workspace=ws)
    C2 = A_.alch_gemm(M, N, terms, a_k, b_k, workspace=ws)
    torch.cuda.synchronize()
    assert rel_err(to_np(C0), ref) < 6e-3 and rel_err(to_np(C1), ref) < 6e-3
    assert torch.equal(C1, C2)


def test_gemm_random_shapes_with_scratch():
    # seeded random sizes around the thresholds of the split (tile counts near 128, 256, 384; short and long
    # contractions; ragged edges), all three layouts, one or two operand pairs, with and without accumulate
    import paper_2503_01066_amd as A_
    rng = np.random.default_rng(2024)
    ws = torch.empty(A_.lib().alch_gemm_workspace_bytes(), dtype=torch.uint8, device="cuda")
    for case in range(14):
        a_k, b_k = [(True, False), (False, False), (True, True)][case % 3]
        tm, tn = int(rng.integers(1, 26)), int(rng.integers(1, 26))
        M = tm * 256 - int(rng.integers(0, 32)) * 8
        N = tn * 256 - int(rng.integers(0, 32)) * 8
        Ks = [int(rng.integers(2, 40)) * 64 for _ in range(int(rng.integers(1, 3)))]
        acc = bool(rng.integers(0, 2))
        terms, ref = [], 0.0
        for K in Ks:
            A, B, r = operands(rng, M, N, K, a_k, b_k, "bf16")
            terms.append((to_dev(A, "bf16"), to_dev(B, "bf16"), K))
            ref = ref + r
        C0 = synth.quantize(rng.standard_normal((M, N)).astype(np.float32) * 20, "bf16")
        C = to_dev(C0, "bf16")
        A_.alch_gemm(M, N, terms, a_k, b_k, out=C, accumulate=acc, workspace=ws)
        torch.cuda.synchronize()
        want = ref + C0 if acc else ref
        assert rel_err(to_np(C), want) < 6e-3, (case, M, N, Ks, a_k, b_k, acc)


@pytest.mark.parametrize("a_k,b_k", [(True, False), (False, False), (True, True)])
def test_gemm_operands_as_column_slices_of_wider_buffers(a_k, b_k):
    # row strides larger than the rows (operands are column ranges of fused buffers, as dQ|dK|dV or G|U are), a row
    # count that leaves the lower half of the last 256-row tile partly empty, three operand pairs of unequal length
    import paper_2503_01066_amd as A_
    rng = np.random.default_rng(77)
    M, N, Ks = 392, 520, [64, 320, 1024]
    ws = torch.empty(A_.lib().alch_gemm_workspace_bytes(), dtype=torch.uint8, device="cuda")
    terms, ref = [], 0.0
    for i, K in enumerate(Ks):
        A, B, r = operands(rng, M, N, K, a_k, b_k, "bf16")
        pa, pb = 8 * (i + 1), 64 * i + 8
        Aw = np.zeros((A.shape[0], A.shape[1] + 2 * pa), A.dtype); Aw[:, pa:pa + A.shape[1]] = A
        Bw = np.zeros((B.shape[0], B.shape[1] + 2 * pb), B.dtype); Bw[:, pb:pb + B.shape[1]] = B
        terms.append((to_dev(Aw, "bf16")[:, pa:pa + A.shape[1]], to_dev(Bw, "bf16")[:, pb:pb + B.shape[1]], K))
        ref = ref + r
    for w in (None, ws):
        C = A_.alch_gemm(M, N, terms, a_k, b_k, workspace=w)
        torch.cuda.synchronize()
        assert rel_err(to_np(C), ref) < 6e-3, (a_k, b_k, w is None)


@pytest.mark.parametrize("a_k,b_k", [(True, False), (False, False)])
def test_gemm_token_indexed_operand_of_more_than_2_gib(a_k, b_k):
    # an operand whose rows are tokens, 40,000 rows of a [*, 28672] buffer (2.3 GB): beyond what one launch of the
    # matrix-core kernel addresses; the product is cut into row bands (data gradient) or contraction bands
    # (weight gradient) of that kernel instead of dropping to the plain fp32 kernel
    import paper_2503_01066_amd as A_
    rng = np.random.default_rng(5)
    T, wide = 40000, 28672
    big = torch.zeros((T, wide), dtype=torch.bfloat16, device="cuda")
    if a_k:      # C[T, 256] = A[T, 128] B[128, 256], A a column slice of the big buffer
        M, N, K = T, 256, 128
        A, B, ref = operands(rng, M, N, K, True, False, "bf16")
        big[:, 64:64 + K] = to_dev(A, "bf16")
        terms = [(big[:, 64:64 + K], to_dev(B, "bf16"), K)]
    else:        # C[256, 128] (+)= A[T, 256]^T B[T, 128], A a column slice of the big buffer, contraction over tokens
        M, N, K = 256, 128, T
        A, B, ref = operands(rng, M, N, K, False, False, "bf16")
        big[:, 64:64 + M] = to_dev(A, "bf16")
        terms = [(big[:, 64:64 + M], to_dev(B, "bf16"), K)]
    A_.alch_trace_enable(True)
    C = A_.alch_gemm(M, N, terms, a_k, b_k)
    torch.cuda.synchronize()
    A_.alch_trace_enable(False)
    kinds = [r[0] for r in A_.alch_trace_collect()]
    assert kinds and all(k == "gemm_mfma" for k in kinds) and len(kinds) >= 2, kinds
    assert rel_err(to_np(C), ref) < (6e-3 if a_k else 1.2e-2)   # contraction bands round once per band
