"""GPU parity of the stage-load GEMM (bf16 MFMA, fp32 accumulate) against the fp64 oracle."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2409_06941_amd as fr          # noqa: E402
from oracle.gemm import gemm_nt            # noqa: E402
from workloads import gemm_inputs          # noqa: E402


def _to_dev_bf16(x32):
    bits = gemm_inputs.bf16_bits(x32).view(np.int16)
    return torch.from_numpy(bits).cuda()


# from two tiles to more than two tiles per CU; tile counts that are and are not multiples of the 8 XCDs
@pytest.mark.parametrize("M,N,K", [(256, 256, 64), (256, 512, 192), (768, 256, 4096), (512, 1280, 320),
                                   (2048, 8192, 128), (1024, 16384 + 256, 192)])
def test_gemm_matches_oracle(M, N, K):
    print("gemm", M, N, K, flush=True)
    a, b = gemm_inputs.operands(M, N, K, seed=M + N + K)
    A, B = _to_dev_bf16(a), _to_dev_bf16(b)
    Cm = torch.zeros((M, N), dtype=torch.int16, device="cuda")
    fr.fr_gemm_bf16(A, B, Cm, M, N, K, torch.cuda.current_stream())
    torch.cuda.synchronize()
    got = gemm_inputs.bits_to_f32(Cm.cpu().numpy().view(np.uint16)).astype(np.float64)
    want = gemm_nt(a, b)
    # result = bf16 rounding (relative 2^-8 at most, half an ulp of 8 bits) of an fp32-accumulated sum whose own
    # error is bounded by K * 2^-24 * sum|a||b| <= K * 2^-24 * K (|a|, |b| < 1)
    bound = np.abs(want) * 2.0 ** -8 + K * K * 2.0 ** -24 + 1e-30
    assert np.all(np.abs(got - want) <= bound)
    # and it must be the nearest bf16 for nearly every entry (loose accumulation differences aside)
    nearest = gemm_inputs.bf16_round(want.astype(np.float32)).astype(np.float64)
    assert np.mean(got == nearest) > 0.98


def test_identity_and_shape_errors():
    M = N = K = 256
    a, _ = gemm_inputs.operands(M, N, K, seed=1)
    eye = np.eye(N, K, dtype=np.float32)
    A, B = _to_dev_bf16(a), _to_dev_bf16(eye)
    Cm = torch.zeros((M, N), dtype=torch.int16, device="cuda")
    fr.fr_gemm_bf16(A, B, Cm, M, N, K, torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert np.array_equal(Cm.cpu().numpy().view(np.uint16), gemm_inputs.bf16_bits(a))     # exact
    for shape in [(250, 256, 64), (256, 100, 64), (256, 256, 72), (0, 256, 64)]:
        with pytest.raises(fr.FreeRideError) as e:
            fr.fr_gemm_bf16(A, B, Cm, *shape, torch.cuda.current_stream())
        assert e.value.code == fr.FR_ERR_ARG


def test_gpt_load_bursts_run_and_report_flops():
    layers, h, ffn, T = 2, 512, 2048, 256
    need = fr.Load.fr_load_workspace_bytes(fr.FR_LOAD_GPT, layers, h, ffn, T)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    load = fr.Load(fr.FR_LOAD_GPT, layers, h, ffn, T, workspace=ws, seed=7, stream=torch.cuda.current_stream())
    fp, bp = load.fr_load_flops()
    per_layer = 2 * T * (3 * h * h + h * h + 2 * h * ffn)
    assert fp == layers * per_layer and bp == 2 * fp
    load.fr_load_fp(torch.cuda.current_stream())
    load.fr_load_bp(torch.cuda.current_stream())
    torch.cuda.synchronize()
    load.fr_load_destroy()
    with pytest.raises(fr.FreeRideError):
        fr.Load(fr.FR_LOAD_GPT, layers, h, ffn, T, workspace=ws[: need // 2], seed=7)
