"""The library's host side -- descriptor checks, workspace layouts, launch planning up to the point where a kernel
would be enqueued (csrc/api.hip, csrc/api_block.hip) -- rebuilt with UndefinedBehaviorSanitizer in trap mode on the
host pass and swept with descriptors whose fields take values across the whole int32 range.  Any signed overflow,
bad shift or out-of-range index in that code kills the sweeping process with a trap.  No kernel is launched (tensor
arguments are NULL, so every call that gets past the descriptor checks stops at the pointer checks): CPU only.
The device code and all other objects are the ordinary build's."""
import os
import subprocess
import sys
import textwrap

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


@pytest.fixture(scope="module")
def sanitized_lib(tmp_path_factory):
    from paper_2505_24544_amd import build as bld
    bdir = os.path.join(bld.CSRC, "_build")
    others = [s for s in bld.sources() if s not in ("api.hip", "api_block.hip")]
    if not all(os.path.exists(os.path.join(bdir, s.replace(".hip", ".o"))) for s in others):
        bld.build(verbose=False)
    out = tmp_path_factory.mktemp("ubsan")
    objs = [os.path.join(bdir, s.replace(".hip", ".o")) for s in others]
    san = ["-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fsanitize-trap=undefined"]
    for src in ("api.hip", "api_block.hip"):
        obj = str(out / src.replace(".hip", ".o"))
        flags = [f for f in bld.FLAGS if f != "-O3"] + ["-O1", "-g"]
        r = subprocess.run([bld.HIPCC, *flags, *san, "-c", os.path.join(bld.CSRC, src), "-o", obj],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-3000:]
        objs.append(obj)
    lib = str(out / "libbeagle_xattn_ubsan.so")
    r = subprocess.run([bld.HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", *objs, "-o", lib],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    return lib


SWEEP = textwrap.dedent('''
    import itertools, sys, ctypes as C
    sys.path.insert(0, sys.argv[2])
    import paper_2505_24544_amd.binding as bx
    bx.LIB_PATH = sys.argv[1]
    L = bx.lib()
    EDGE = (-2**31, -1, 0, 1, 3, 8, 64, 128, 4096, 2**20 + 1, 2**30, 2**30 + 1, 2**31 - 1)
    BASE = dict(batch=2, seq_q=64, seq_kv=64, hidden=256, n_q_heads=2, n_kv_heads=1, head_dim=128, block_size=4,
                block_offset=1, io_dtype=bx.BEAGLE_BF16, flags=0, total_q=0, total_kv=0)
    WS = (bx.BEAGLE_WS_FWD, bx.BEAGLE_WS_BWD, bx.BEAGLE_WS_DRAFT, bx.BEAGLE_WS_APPEND, bx.BEAGLE_WS_BWD_SIM, 17, -1)
    n = 0

    def poke(desc):
        """Every entry point that reads a descriptor; NULL tensors stop each call before anything is enqueued."""
        global n
        n += 1
        for w in WS:
            L.beagle_xattn_workspace_bytes(C.byref(desc), w)
        for w in (0, 1, 2, 3, 9):
            for f in (64, 11008, 2**31 - 1, -5):
                L.beagle_xattn_block_workspace_bytes(C.byref(desc), f, w)
        z = None
        bx.beagle_xattn_fwd(desc, z, z, z, z, z, z, z, z, z, z, z, z, z, check=False, workspace_bytes=1 << 40, stream=0)
        bx.beagle_xattn_bwd(desc, *([z] * 18), z, check=False, workspace_bytes=1 << 40, stream=0)
        bx.beagle_xattn_draft_step(desc, z, z, z, z, z, z, z, z, check=False, workspace_bytes=1 << 40, stream=0)
        bx.beagle_xattn_draft_step_tree(desc, z, z, z, z, z, 5, z, 1, z, z, z, check=False, workspace_bytes=1 << 40, stream=0)
        bx.beagle_xattn_draft_step_prepared(desc, z, z, z, z, z, 5, z, 1, z, z, z, check=False, workspace_bytes=1 << 40, stream=0)
        bx.beagle_xattn_prepare_weights(desc, check=False, stream=0)
        bx.beagle_xattn_kv_append_prepared(desc, z, z, z, z, z, 3, check=False, stream=0)
        bx.beagle_xattn_block_kv_append_prepared(desc, bx.make_block_params(64, 1e-5), bx.make_block_decode_weights(), z, z, z, 3,
                                                 check=False, stream=0)
        bx.beagle_xattn_kv_append(desc, z, z, z, z, z, 3, z, check=False, workspace_bytes=1 << 40, stream=0)
        for ffn in (64, 11008, 2**31 - 64):
            p = bx.make_block_params(ffn, 1e-5)
            bx.beagle_xattn_block_draft_step(desc, p, z, z, z, 5, z, 1, z, z, z, check=False, workspace_bytes=1 << 40, stream=0)
            bx.beagle_xattn_block_draft_step_prepared(desc, p, bx.make_block_decode_weights(), z, z, z, 5, z, 1, z, z, z,
                                                      check=False, workspace_bytes=1 << 40, stream=0)
            bx.beagle_xattn_block_prepare_weights(desc, p, bx.make_block_decode_weights(), check=False, stream=0)
            bx.beagle_xattn_block_fwd(desc, p, z, z, z, bx.make_block_saved(), z, check=False, workspace_bytes=1 << 40, stream=0)
            bx.beagle_xattn_block_bwd(desc, p, z, z, z, bx.make_block_saved(), bx.make_block_grads(), z, check=False,
                                      workspace_bytes=1 << 40, stream=0)
        # the host-side mask helpers write S (or S*L, or tiles) integers: only where that is small
        if 0 < desc.seq_q <= 4096 and 0 < desc.seq_kv <= 4096:
            S, Lk = desc.seq_q, desc.seq_kv
            lim = (C.c_int32 * S)()
            L.beagle_xattn_mask_row_limit(C.byref(desc), lim)
            if S * Lk <= 1 << 16:
                m = (C.c_uint8 * (S * Lk))()
                L.beagle_xattn_mask_dense(C.byref(desc), m)
            for tq, tk in ((128, 64), (1, 1), (7, 5), (2**31 - 1, 2**31 - 1), (0, 4), (-3, 8)):
                if tq > 0 and tk > 0 and ((S + tq - 1) // tq) * ((Lk + tk - 1) // tk) <= 1 << 16:
                    cls = (C.c_uint8 * (((S + tq - 1) // tq) * ((Lk + tk - 1) // tk)))()
                    L.beagle_xattn_tile_map(C.byref(desc), tq, tk, cls)
                elif tq <= 0 or tk <= 0:
                    L.beagle_xattn_tile_map(C.byref(desc), tq, tk, None)

    # one field at a time through every edge value, for both dtypes and the flag combinations
    for dtype in (bx.BEAGLE_BF16, bx.BEAGLE_F32):
        for flags in (0, bx.BEAGLE_FLAG_NEED_DXKV | bx.BEAGLE_FLAG_ROPE, 0xffffffff):
            for field in ("batch", "seq_q", "seq_kv", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "block_size",
                          "block_offset", "total_q", "total_kv"):
                for v in EDGE:
                    poke(bx.make_desc(**dict(BASE, io_dtype=dtype, flags=flags & 0xffffffff, **{field: v})))
    # pairs of large fields together: products are where overflow hides
    big = (1, 4096, 2**20, 2**30, 2**31 - 1)
    for a, b, c in itertools.product(big, big, big):
        poke(bx.make_desc(**dict(BASE, batch=1, seq_q=a, seq_kv=b, hidden=c if c % 8 == 0 else 4096, n_q_heads=32,
                                 n_kv_heads=8)))
        poke(bx.make_desc(**dict(BASE, batch=a, seq_q=b, seq_kv=b, hidden=4096, n_q_heads=32, n_kv_heads=32,
                                 block_size=c, block_offset=max(0, c - 1))))
    print("descriptors swept:", n)
''')


def test_descriptor_sweep_under_ubsan(sanitized_lib, tmp_path):
    script = tmp_path / "sweep.py"
    script.write_text(SWEEP)
    r = subprocess.run([sys.executable, str(script), sanitized_lib, ROOT], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, "the sweep died (a trap is an undefined-behaviour report):\n%s\n%s" % (r.stdout[-2000:], r.stderr[-4000:])
    assert "descriptors swept:" in r.stdout
