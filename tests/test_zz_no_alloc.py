"""entro_decode_gemv_static (the entry point that allocates nothing) against entro_decode_gemv.

Two calls in a row on the same GPU, the second on a smaller tensor: the library's static partial-sum
array keeps the first call's contents, and the second result must not depend on them.  Both entry
points run the same kernels, so the outputs are compared bit for bit; the reference call is also held
to the GEMV bar against the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_02380_amd as E
from paper_2505_02380_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(seed, rows, cols, chunk):
    rng = np.random.default_rng(seed)
    sym = np.clip(np.rint(rng.standard_t(5, rows * cols) * 6 + 128), 0, 255).astype(np.uint8)
    ln, code, _ = oracle.codebook_from_symbols(sym, 8)
    stream, off = oracle.encode(sym, ln, code, chunk)
    cb = E.entro_codebook_from_lengths(ln, 8)
    qp = B.QParams(np.float32(0.0123), 131, 8, E.ENTRO_ASYMMETRIC)
    enc = B.EncodedTensor(stream, off, sym.size, chunk, cb, qp, rows, cols)
    xb = (rng.standard_normal(cols).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    y_ref, _ = oracle.gemv(sym, rows, cols, qp.scale, qp.zero_point, xb)
    return enc, xb, y_ref


@pytest.mark.parametrize("y_type", [E.ENTRO_F32, E.ENTRO_BF16])
def test_static_scratch_gemv_matches_the_workspace_form_twice_in_a_row(y_type):
    dtype = torch.float32 if y_type == E.ENTRO_F32 else torch.bfloat16
    # rows of 1536 and 1088 weights in segments of 4096 and 2048: most rows straddle segments
    for seed, rows, cols, chunk in ((1, 640, 1536, 4096), (2, 96, 1088, 2048)):
        enc, xb, y_ref = _case(seed, rows, cols, chunk)
        dt = E.to_device(enc, DEV)
        x = torch.from_numpy(xb.view(np.int16)).to(DEV).view(torch.bfloat16)
        y_ws = torch.zeros(rows + 8, dtype=dtype, device=DEV)
        y_st = torch.zeros(rows + 8, dtype=dtype, device=DEV)
        t_ws = dt.ctensor(y_ws, x)
        need = E.entro_gemv_workspace_bytes(t_ws)
        assert need > 0, "the case must use partial sums"
        ws = torch.zeros(need, dtype=torch.uint8, device=DEV)
        E.entro_decode_gemv(t_ws, y_type, ws)
        E.entro_decode_gemv_static(dt.ctensor(y_st, x), y_type)
        torch.cuda.synchronize()
        assert torch.equal(y_ws.view(torch.int32 if y_type == E.ENTRO_F32 else torch.int16),
                           y_st.view(torch.int32 if y_type == E.ENTRO_F32 else torch.int16))
        y = y_st[:rows].float().cpu().numpy().astype(np.float64)
        rms = np.sqrt(np.mean(y_ref ** 2))
        tol = 1e-3 if y_type == E.ENTRO_F32 else 4e-3          # bf16 y: half an ulp is 2^-9
        assert np.max(np.abs(y - y_ref) / np.maximum(np.abs(y_ref), rms)) <= tol
        assert torch.all(y_st[rows:] == 0)


def test_static_scratch_gemv_rejects_more_segments_than_the_array_holds():
    # a descriptor is enough: the size check comes before anything touches the buffers' contents
    enc, xb, _ = _case(3, 8, 1536, 4096)
    dt = E.to_device(enc, DEV)
    x = torch.from_numpy(xb.view(np.int16)).to(DEV).view(torch.bfloat16)
    y = torch.zeros(16, dtype=torch.float32, device=DEV)
    t = dt.ctensor(y, x)
    t.rows, t.cols = 1 << 18, 1536
    t.n = t.rows * t.cols                      # 96 K segments of 4096 > 65536
    with pytest.raises(E.EntroError) as err:
        E.entro_decode_gemv_static(t, E.ENTRO_F32)
    assert err.value.status == B.ENTRO_ERR_CAPACITY
