"""Helpers of the GPU parity tests: move synthetic tensors to the device, call the C ABI through
the binding, bring results back as numpy.  No method arithmetic here."""
import numpy as np
import torch

import paper_2509_21302_amd as q

DEV = "cuda:0"


def to_dev(a):
    """Synthetic tensor -> device tensor.  uint16 arrays are bf16 bit patterns."""
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(a).to(DEV)


def bf16_bits(t):
    """device bf16 tensor -> numpy uint16 bit patterns"""
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def gpu_prep(W, X_cal, signs, alpha=0.5):
    """qvggt_rotated_col_absmax + qvggt_prep_weights.  Returns dict of device tensors."""
    Wd, sd = to_dev(W), to_dev(signs)
    N, K = Wd.shape
    a = None
    if X_cal is not None:
        a = torch.empty(K, dtype=torch.float32, device=DEV)
        q.qvggt_rotated_col_absmax(to_dev(X_cal), sd, a)
    Wq = torch.empty(N, K // 2, dtype=torch.uint8, device=DEV)
    sw = torch.empty(N, dtype=torch.float32, device=DEV)
    inv = torch.empty(K, dtype=torch.float32, device=DEV)
    q.qvggt_prep_weights(Wd, a, sd, alpha, Wq, sw, inv)
    return dict(Wq=Wq, sw=sw, inv=inv, signs=sd, a=a, N=N, K=K)


def gpu_rsq(Xd, signs_d, inv_d):
    M, K = Xd.shape
    Xq = torch.empty(M, K // 2, dtype=torch.uint8, device=DEV)
    sx = torch.empty(M, dtype=torch.float32, device=DEV)
    q.qvggt_rotate_smooth_quant(Xd, signs_d, inv_d, Xq, sx)
    return Xq, sx


def gpu_ln_rsq(Xd, gamma_d, beta_d, eps, signs_d, inv_d):
    M, K = Xd.shape
    Xq = torch.empty(M, K // 2, dtype=torch.uint8, device=DEV)
    sx = torch.empty(M, dtype=torch.float32, device=DEV)
    q.qvggt_layernorm_rotate_smooth_quant(Xd, gamma_d, beta_d, eps, signs_d, inv_d, Xq, sx)
    return Xq, sx


def gpu_rsq_asym(Xd, signs_d, inv_d):
    """Affine activation codes: returns (Xq nibbles holding u - 8, steps, zero points)."""
    M, K = Xd.shape
    Xq = torch.empty(M, K // 2, dtype=torch.uint8, device=DEV)
    sx = torch.empty(M, dtype=torch.float32, device=DEV)
    zx = torch.empty(M, dtype=torch.float32, device=DEV)
    q.qvggt_rotate_smooth_quant_asym(Xd, signs_d, inv_d, Xq, sx, zx)
    return Xq, sx, zx


def gpu_code_sums(Wq, N, K):
    s = torch.empty(N, dtype=torch.float32, device=DEV)
    q.qvggt_weight_code_sums(Wq, N, K, s)
    return s


def gpu_rsq_static(Xd, signs_d, inv_d, step_d, per_token):
    M, K = Xd.shape
    Xq = torch.empty(M, K // 2, dtype=torch.uint8, device=DEV)
    sx = torch.empty(M, dtype=torch.float32, device=DEV)
    q.qvggt_rotate_smooth_quant_static(Xd, signs_d, inv_d, step_d, per_token, Xq, sx)
    return Xq, sx


def gpu_unpack(packed, K):
    rows = packed.shape[0]
    codes = torch.empty(rows, K, dtype=torch.int8, device=DEV)
    q.qvggt_unpack_int4(packed, codes)
    return codes.cpu().numpy()


def gpu_pack(codes_np):
    c = torch.from_numpy(np.ascontiguousarray(codes_np, dtype=np.int8)).to(DEV)
    rows, K = c.shape
    packed = torch.empty(rows, K // 2, dtype=torch.uint8, device=DEV)
    q.qvggt_pack_int4(c, packed)
    return packed


_gelu_table = None


def gelu_table():
    """the device table of qvggt_gelu_table (built once per test process)"""
    global _gelu_table
    if _gelu_table is None:
        _gelu_table = torch.empty(q.qvggt_gelu_table_bytes(), dtype=torch.uint8, device=DEV)
        q.qvggt_gelu_table(_gelu_table)
    return _gelu_table


def codes_to_e2m3(packed, rows, K, out, expect_clean=True):
    """qvggt_codes_to_e2m3 with its counter of codes -8 (which have no E2M3 value): returns the count, 0 expected by default"""
    cnt = torch.zeros(1, dtype=torch.int32, device=DEV)
    q.qvggt_codes_to_e2m3(packed, rows, K, out, cnt)
    n = int(cnt.item())
    assert n == 0 or not expect_clean, f"{n} codes -8 in a buffer that should hold none"
    return n


def gpu_linear(Xd, prep, bias_d):
    M, K = Xd.shape
    N = prep["N"]
    Y = torch.empty(M, N, dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(q.qvggt_workspace_bytes(M, N, K), dtype=torch.uint8, device=DEV)
    q.qvggt_linear(Xd, prep["signs"], prep["inv"], prep["Wq"], prep["sw"], bias_d, Y, ws)
    return Y


# ---- the 8-bit / 6-bit settings (int8 codes)
def gpu_layout_int8(codes, to_library):
    """numpy or device int8 [rows, K] -> device int8 [rows, K] in the other order"""
    c = codes if torch.is_tensor(codes) else torch.from_numpy(np.ascontiguousarray(codes, dtype=np.int8)).to(DEV)
    out = torch.empty_like(c)
    q.qvggt_layout_int8(c, out, to_library)
    return out


def gpu_prep_i8(W, X_cal, signs, bits, alpha=0.5):
    Wd, sd = to_dev(W), to_dev(signs)
    N, K = Wd.shape
    a = None
    if X_cal is not None:
        a = torch.empty(K, dtype=torch.float32, device=DEV)
        q.qvggt_rotated_col_absmax(to_dev(X_cal), sd, a)
    Wq = torch.empty(N, K, dtype=torch.int8, device=DEV)
    sw = torch.empty(N, dtype=torch.float32, device=DEV)
    inv = torch.empty(K, dtype=torch.float32, device=DEV)
    q.qvggt_prep_weights_i8(Wd, a, sd, alpha, bits, Wq, sw, inv)
    return dict(Wq=Wq, sw=sw, inv=inv, signs=sd, a=a, N=N, K=K, bits=bits)


def gpu_rsq_i8(Xd, signs_d, inv_d, bits):
    M, K = Xd.shape
    Xq = torch.empty(M, K, dtype=torch.int8, device=DEV)
    sx = torch.empty(M, dtype=torch.float32, device=DEV)
    q.qvggt_rotate_smooth_quant_i8(Xd, signs_d, inv_d, bits, Xq, sx)
    return Xq, sx


def gpu_linear_i8(Xd, prep, bias_d):
    M, K = Xd.shape
    N = prep["N"]
    Y = torch.empty(M, N, dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(q.qvggt_workspace_bytes_i8(M, N, K), dtype=torch.uint8, device=DEV)
    q.qvggt_linear_i8(Xd, prep["signs"], prep["inv"], prep["bits"], prep["Wq"], prep["sw"], bias_d, Y, ws)
    return Y


# ---- the acceptance criteria of the quantized path -----------------------------------------
CODE_MISMATCH_FRACTION = 1e-4     # activation codes may differ by one step on at most 0.01 % of elements
SCALE_RTOL = 1e-5                 # fp32 butterflies and scaling against the fp64 oracle
Y_REL_FRO = 1e-2                  # final bf16 output, relative Frobenius error


def check_codes(got, want, what=""):
    d = np.abs(got.astype(np.int16) - want.astype(np.int16))
    assert d.max(initial=0) <= 1, f"{what}: a code differs by {d.max()}"
    frac = float((d != 0).mean()) if d.size else 0.0
    assert frac <= CODE_MISMATCH_FRACTION, f"{what}: {frac:.3e} of the codes differ (allowed {CODE_MISMATCH_FRACTION})"
    return frac


def check_scales(got, want, what=""):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    err = np.abs(got - want) / np.maximum(np.abs(want), 1e-300)
    err[want == 0] = np.abs(got[want == 0])
    assert err.max(initial=0) <= SCALE_RTOL, f"{what}: scale rel err {err.max():.3e}"


def rel_fro(got_bits, want_bits):
    g = (np.asarray(got_bits, np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    w = (np.asarray(want_bits, np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return float(np.linalg.norm(g - w) / max(np.linalg.norm(w), 1e-300))


def decode_e2m3_rows(buf, rows, K):
    """E2M3 blocks -> value at every position of the packed row, from the format's definition: sign, 2 exponent bits (bias 1),
    3 mantissa bits; exponent 0 is subnormal (m / 8).  Unit s of row r starts at ((r / 128) * (K / 64) + s) * 6144 + (r % 128) * 48."""
    out = np.zeros((rows, K), dtype=np.float64)
    r = np.arange(rows)
    for s in range(K // 64):
        start = ((r // 128) * (K // 64) + s) * 6144 + (r % 128) * 48
        unit = buf[start[:, None] + np.arange(48)[None, :]]
        for h in range(2):
            blob = np.concatenate([unit[:, 16 * h: 16 * h + 16], unit[:, 32 + 8 * h: 40 + 8 * h]], axis=1)     # 24 bytes
            bits = np.unpackbits(blob, axis=1, bitorder="little")                                            # [rows, 192]
            for i in range(32):
                f = bits[:, 6 * i: 6 * i + 6].astype(np.int64)
                m = f[:, 0] + 2 * f[:, 1] + 4 * f[:, 2]
                e = f[:, 3] + 2 * f[:, 4]
                mag = np.where(e == 0, m / 8.0, 2.0 ** (e - 1) * (1 + m / 8.0))
                out[:, 64 * s + 32 * h + i] = np.where(f[:, 5] == 1, -mag, mag)
    return out


def report(name, **values):
    """Measured figures of a GPU test (achieved errors and mismatch fractions, not pass / fail): printed, and appended as one
    JSON line to measured.jsonl in the folder QVGGT_MEASURED_DIR names (default: the run's output folder at the repository root)
    when that folder exists; the bars of the fused-neighbour tests were set from these figures."""
    import json
    import os
    line = json.dumps(dict(test=name, **{k: (float(v) if isinstance(v, (float, np.floating)) else v) for k, v in values.items()}))
    print("measured:", line)
    d = os.environ.get("QVGGT_MEASURED_DIR") or os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out")
    if os.path.isdir(d):
        with open(os.path.join(d, "measured.jsonl"), "a") as f:
            f.write(line + "\n")
