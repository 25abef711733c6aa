"""The C-ABI library loads without a GPU and exports every symbol the header declares."""
import ctypes
import os
import re

import paper_2406_16747_amd as spk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "sparsek.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sparsek_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    if not os.path.exists(spk.lib_path()):
        from paper_2406_16747_amd import build

        build.build()
    L = ctypes.CDLL(spk.lib_path())
    names = declared_symbols()
    assert len(names) >= 12
    for name in names:
        assert hasattr(L, name), name


def test_argument_validation_needs_no_gpu():
    L = spk.lib()
    cfg = spk.SparsekCfg(B=1, H=2, Gu=1, n=16, d=64, k=4, w=4, dtype=spk.BF16, gate_mode=0, softmax_scale=1.0)
    null = ctypes.c_void_p(0)
    one_ = ctypes.c_void_p(256)  # never dereferenced: validation fails first
    assert L.sparsek_mask(ctypes.byref(cfg), null, null, null, null, 0, null) == -1
    assert L.sparsek_mask_workspace_bytes(ctypes.byref(cfg)) > 0
    flag = ctypes.c_int32(7)
    assert L.sparsek_mask_status(ctypes.byref(cfg), null, 1 << 20, ctypes.byref(flag), null) == -1
    assert L.sparsek_mask_status(ctypes.byref(cfg), one_, 8, ctypes.byref(flag), null) == -3
    # k or w far beyond any sequence length are refused, not wrapped around
    for kw in ((2 ** 31 - 1, 4), (4, 2 ** 31 - 1), (2 ** 31 - 1, 2 ** 31 - 1)):
        big = spk.SparsekCfg(B=1, H=2, Gu=1, n=16, d=64, k=kw[0], w=kw[1], dtype=spk.BF16, gate_mode=0, softmax_scale=1.0)
        assert L.sparsek_mask_workspace_bytes(ctypes.byref(big)) == 0
        assert L.sparsek_attn_fwd(ctypes.byref(big), *([one_] * 8), one_, 1 << 20, null) == -2
    bad = spk.SparsekCfg(B=1, H=2, Gu=3, n=16, d=64, k=4, w=4, dtype=spk.BF16, gate_mode=0, softmax_scale=1.0)
    assert L.sparsek_mask_workspace_bytes(ctypes.byref(bad)) == 0
    one = ctypes.c_void_p(256)  # never dereferenced: validation fails first
    assert L.sparsek_mask(ctypes.byref(bad), one, one, one, one, 1 << 20, null) == -1
    bad = spk.SparsekCfg(B=1, H=2, Gu=1, n=16, d=64, k=0, w=0, dtype=spk.BF16, gate_mode=0, softmax_scale=1.0)
    assert L.sparsek_attn_fwd(ctypes.byref(bad), *([one] * 8), one, 1 << 20, null) == -1
    bad = spk.SparsekCfg(B=1, H=2, Gu=1, n=16, d=96 + 1, k=1, w=0, dtype=spk.BF16, gate_mode=0, softmax_scale=1.0)
    assert L.sparsek_attn_fwd(ctypes.byref(bad), *([one] * 8), one, 1 << 20, null) == -2
    assert L.sparsek_attn_fwd(ctypes.byref(cfg), *([one] * 8), one, 8, null) == -3
    assert b"workspace" in L.sparsek_strerror(-3)
    # importance scores
    from paper_2406_16747_amd.binding import SparsekScoresCfg

    sc = SparsekScoresCfg(B=2, n=100, D=768, dtype=spk.BF16, norm=1, slope=0.0, norm_eps=1e-5)
    assert L.sparsek_scores_workspace_bytes(ctypes.byref(sc)) >= 2 * 100 * 8
    assert L.sparsek_scores(ctypes.byref(sc), null, one, one, one, 1 << 20, null) == -1
    assert L.sparsek_scores(ctypes.byref(sc), one, one, one, one, 8, null) == -3
    bad = SparsekScoresCfg(B=2, n=100, D=100, dtype=spk.BF16, norm=0, slope=0.0, norm_eps=1e-5)
    assert L.sparsek_scores(ctypes.byref(bad), one, one, one, one, 1 << 20, null) == -2  # D % 8
    bad = SparsekScoresCfg(B=2, n=100, D=768, dtype=spk.BF16, norm=1, slope=0.0, norm_eps=0.0)
    assert L.sparsek_scores(ctypes.byref(bad), one, one, one, one, 1 << 20, null) == -1  # eps must be > 0
    bad = SparsekScoresCfg(B=2, n=100, D=768, dtype=spk.BF16, norm=2, slope=0.0, norm_eps=1e-5)
    assert L.sparsek_scores(ctypes.byref(bad), one, one, one, one, 1 << 20, null) == -1
    # gate modes 0..3 are valid, 4 is not
    bad = spk.SparsekCfg(B=1, H=2, Gu=1, n=16, d=64, k=4, w=4, dtype=spk.BF16, gate_mode=4, softmax_scale=1.0)
    assert L.sparsek_attn_fwd(ctypes.byref(bad), *([one] * 8), one, 1 << 20, null) == -1
    # chunk-wise recurrent prefill
    from paper_2406_16747_amd.binding import SparsekChunkCfg, SparsekDecodeCfg

    cc = SparsekChunkCfg(B=1, H=2, Gu=1, d=64, k=8, w=8, cand_cap=0, chunk_max=256, dtype=spk.BF16, gate_mode=0,
                         softmax_scale=1.0)
    sb, wb = L.sparsek_chunk_state_bytes(ctypes.byref(cc)), L.sparsek_chunk_workspace_bytes(ctypes.byref(cc))
    assert sb > 0 and wb > 0
    assert L.sparsek_chunk_init(ctypes.byref(cc), null, sb, null) == -1
    assert L.sparsek_chunk_init(ctypes.byref(cc), one, 8, null) == -3
    assert L.sparsek_chunk_prefill(ctypes.byref(cc), one, sb, 0, one, one, one, one, one, one, wb, null) == -1  # c < 1
    assert L.sparsek_chunk_prefill(ctypes.byref(cc), one, sb, 257, one, one, one, one, one, one, wb, null) == -1  # c > chunk_max
    assert L.sparsek_chunk_prefill(ctypes.byref(cc), one, sb, 16, one, one, one, one, one, one, 8, null) == -3
    bad = SparsekChunkCfg(B=1, H=2, Gu=1, d=4, k=8, w=8, cand_cap=0, chunk_max=256, dtype=spk.BF16, gate_mode=0,
                          softmax_scale=1.0)
    assert L.sparsek_chunk_state_bytes(ctypes.byref(bad)) == 0  # rows of 8 bytes: not a multiple of 16
    dc = SparsekDecodeCfg(B=1, H=2, Gu=1, d=64, k=8, w=8, cand_cap=0, dtype=spk.BF16, gate_mode=0, softmax_scale=1.0)
    db = L.sparsek_decode_state_bytes(ctypes.byref(dc))
    assert L.sparsek_chunk_to_decode(ctypes.byref(cc), one, sb, 15, one, wb, ctypes.byref(dc), one, db, null) == -2  # < k + w
    dc.k = 9
    assert L.sparsek_chunk_to_decode(ctypes.byref(cc), one, sb, 100, one, wb, ctypes.byref(dc), one, db, null) == -1
    # attention backward: 9 tensors in, 3 out, a workspace
    assert L.sparsek_attn_bwd_workspace_bytes(ctypes.byref(cfg)) > 0
    assert L.sparsek_attn_bwd(ctypes.byref(cfg), *([one] * 9), one, one, null, one, 1 << 30, null) == -1  # dv null
    assert L.sparsek_attn_bwd(ctypes.byref(cfg), *([one] * 9), one, one, one, one, 8, null) == -3
    bad = spk.SparsekCfg(B=1, H=2, Gu=1, n=16, d=64, k=4, w=4, dtype=spk.BF16, gate_mode=4, softmax_scale=1.0)
    assert L.sparsek_attn_bwd(ctypes.byref(bad), *([one] * 9), one, one, one, one, 1 << 30, null) == -1
    # backward of a chunk (bf16, d = 64 / 128 only)
    cc = SparsekChunkCfg(B=1, H=2, Gu=1, d=64, k=8, w=8, cand_cap=0, chunk_max=256, dtype=spk.BF16, gate_mode=0,
                         softmax_scale=1.0)
    wb, bb = L.sparsek_chunk_workspace_bytes(ctypes.byref(cc)), L.sparsek_chunk_bwd_workspace_bytes(ctypes.byref(cc))
    assert bb > 0
    assert L.sparsek_chunk_bwd(ctypes.byref(cc), 16, one, one, one, one, wb, one, one, one, null, one, bb, null) == -1
    assert L.sparsek_chunk_bwd(ctypes.byref(cc), 0, one, one, one, one, wb, one, one, one, one, one, bb, null) == -1
    assert L.sparsek_chunk_bwd(ctypes.byref(cc), 16, one, one, one, one, wb, one, one, one, one, one, 8, null) == -3
    f32 = SparsekChunkCfg(B=1, H=2, Gu=1, d=64, k=8, w=8, cand_cap=0, chunk_max=256, dtype=spk.F32, gate_mode=0,
                          softmax_scale=1.0)
    assert L.sparsek_chunk_bwd_workspace_bytes(ctypes.byref(f32)) == 0
    assert L.sparsek_chunk_bwd(ctypes.byref(f32), 16, one, one, one, one, 1 << 30, one, one, one, one, one, 1 << 30, null) == -2
    # the one-call backward
    assert L.sparsek_bwd_workspace_bytes(ctypes.byref(cfg)) > L.sparsek_attn_bwd_workspace_bytes(ctypes.byref(cfg))
    assert L.sparsek_bwd(ctypes.byref(cfg), *([one] * 9), one, one, one, null, one, 1 << 30, null) == -1  # du null
    assert L.sparsek_bwd(ctypes.byref(cfg), *([one] * 9), one, one, one, one, one, 8, null) == -3


def test_toolchain_record_and_m0_check():
    """Three kernels set the M0 register from inline assembly (direct-to-LDS loads the compiler does not track), which
    is sound only while the compiler keeps nothing of its own in M0 inside those kernels.  The build checks the
    generated assembly for that and records the compiler; a compiler other than the validated one calls for a fresh
    run of the GPU parity tests (then update VALIDATED_HIPCC in build.py)."""
    import json

    from paper_2406_16747_amd import build

    if not os.path.exists(build.SIDECAR) or os.path.getmtime(build.SIDECAR) < os.path.getmtime(spk.lib_path()) - 60:
        build.build()
    rec = json.load(open(build.SIDECAR))
    assert rec["m0_check"] == "ok"
    loads = rec["untracked_direct_to_lds_loads"]
    assert set(loads) == {"attn_fwd.hip", "mask_bwd.hip", "attn_bwd.hip"}, loads
    assert rec["hipcc_version"][0].startswith(build.VALIDATED_HIPCC), (
        "libsparsek was built with %r, its hand-written M0 handling was validated with %r: run the GPU parity tests "
        "with this compiler and update VALIDATED_HIPCC" % (rec["hipcc_version"][0], build.VALIDATED_HIPCC))
    # the checker itself: a kernel that mixes hand-written and compiler-managed M0 is refused
    import tempfile

    bad = "k1:\n;;#ASMSTART\ns_mov_b32 m0, s3\ns_nop 0\nglobal_load_lds_dwordx4 v1, s[2:3]\n;;#ASMEND\ns_mov_b32 m0, s9\n.Lfunc_end0:\n"
    good = "k1:\n;;#ASMSTART\ns_mov_b32 m0, s3\ns_nop 0\nglobal_load_lds_dwordx4 v1, s[2:3]\n;;#ASMEND\n.Lfunc_end0:\nk2:\ns_mov_b32 m0, s9\n.Lfunc_end1:\n"
    with tempfile.NamedTemporaryFile("w", suffix=".s", delete=False) as f:
        f.write(bad)
    try:
        build.check_m0(f.name)
        raise AssertionError("a mixed kernel was accepted")
    except RuntimeError:
        pass
    open(f.name, "w").write(good)
    assert build.check_m0(f.name) == {"k1": 1}
    os.remove(f.name)
