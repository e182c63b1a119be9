"""Helpers shared by the GPU parity tests (comparison only; no method arithmetic)."""
import numpy as np
import torch

import paper_2605_18739_amd as nv


def dev_bf16(bits_np):
    return nv.bf16_from_bits(bits_np, "cuda")


def host_q(t):
    """NVFP4Tensor on the device -> (codes, scales, global_scale) numpy."""
    torch.cuda.synchronize()
    return t.codes.cpu().numpy(), t.scales.cpu().numpy(), np.float32(t.global_scale.cpu().numpy()[0])


def assert_q_equal(gpu_t, oq, what=""):
    codes, scales, gs = host_q(gpu_t)
    assert gs.view(np.uint32) == np.float32(oq.global_scale).view(np.uint32), \
        f"{what}: global scale {gs!r} vs oracle {oq.global_scale!r}"
    bad_s = np.argwhere(scales != oq.scales)
    assert bad_s.size == 0, f"{what}: {len(bad_s)} scale bytes differ, first at {bad_s[0]}: " \
                            f"gpu {scales[tuple(bad_s[0])]:#x} oracle {oq.scales[tuple(bad_s[0])]:#x}"
    bad_c = np.argwhere(codes != oq.codes)
    assert bad_c.size == 0, f"{what}: {len(bad_c)} code bytes differ, first at {bad_c[0]}: " \
                            f"gpu {codes[tuple(bad_c[0])]:#x} oracle {oq.codes[tuple(bad_c[0])]:#x}"


# GEMM tolerance: relative Frobenius error <= 1e-5 and per element |err| <= 2^-15 * sum_k |a_k w_k|
REL_FRO = 1e-5
ELEM = 2.0 ** -15


def assert_gemm_close(y_gpu_f32, Y, S, what=""):
    y = np.asarray(y_gpu_f32, dtype=np.float64)
    err = np.abs(y - Y)
    fro = np.linalg.norm(y - Y) / max(np.linalg.norm(Y), 1e-300)
    worst = (err / np.maximum(S, 1e-300)).max()
    assert fro <= REL_FRO, f"{what}: relative Frobenius error {fro:.3e} > {REL_FRO}"
    assert (err <= ELEM * S + 1e-300).all(), f"{what}: per-element bound violated, worst err/S = {worst:.3e}"
    return fro, worst
