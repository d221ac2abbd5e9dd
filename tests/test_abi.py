"""Host-side checks that need no GPU: the library loads, exports every symbol the header
declares, and its host logic (configuration checks, call order, sizes) behaves as documented."""
import ctypes
import os
import re

import pytest

from paper_2404_18911_amd import binding as B
from paper_2404_18911_amd import inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "kangaroo.h")).read()
    declared = set(re.findall(r"\b(kg_[a-z_0-9]+)\s*\(", hdr))
    declared -= {"kg_ctx"}
    assert declared == set(B.SYMBOLS), declared ^ set(B.SYMBOLS)
    L = B.lib()
    for s in declared:
        assert hasattr(L, s), s


def _create(shape, **over):
    cfg = B.make_config(shape, over.pop("max_seq", 64), over.pop("gamma_max", 6), over.pop("kv_page_tokens", 16))
    for k, v in over.items():
        setattr(cfg, k, v)
    h = ctypes.c_void_p()
    rc = B.lib().kg_create(ctypes.byref(cfg), ctypes.byref(h))
    return rc, h


def test_create_validates_the_configuration():
    shape = I.SHAPES["toy"]
    rc, h = _create(shape)
    assert rc == B.KG_OK and h.value
    B.lib().kg_destroy(h)
    for bad in (dict(exit_layer=0), dict(exit_layer=5), dict(head_dim=48), dict(n_heads=3), dict(gamma_max=8),
                dict(kv_page_tokens=24), dict(kv_page_tokens=256), dict(dtype=2), dict(dtype=0, kv_dtype=1), dict(dtype=0, kv_dtype=2), dict(kv_dtype=3),
                dict(vocab=1000), dict(max_seq=1), dict(max_seq=16 * 129), dict(adapter_kind=4), dict(adapter_kind=-1)):
        rc, h = _create(shape, **bad)
        assert rc == B.KG_EINVAL and not h.value, bad


def test_workspace_sizes_match_the_shape():
    import dataclasses
    L = B.lib()
    cases = [I.SHAPES[n] for n in ("toy", "7b", "33b")] + [dataclasses.replace(I.SHAPES["7b"], adapter=a) for a in (1, 2, 3)]
    for shape in cases:
        rc, h = _create(shape, max_seq=520, kv_page_tokens=128)
        assert rc == B.KG_OK
        wb, kb, sb = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
        assert L.kg_workspace_bytes(h, ctypes.byref(wb), ctypes.byref(kb), ctypes.byref(sb)) == B.KG_OK
        params = shape.n_layers * shape.layer_params() + shape.adapter_params() + 2 * shape.head_params() + shape.d_model
        esz = shape.bytes_per_weight()
        # the tiled arena holds every matrix once (gains as fp32): within 1% of the raw parameter bytes
        assert params * esz <= wb.value <= params * esz * 1.01 + (1 << 20)
        pages = (520 + 127) // 128
        kvb = pages * 128 * (shape.n_layers + 1) * 2 * shape.d_model * (4 if shape.kv_dtype == "f32" else 2)
        assert kb.value == kvb
        assert sb.value > 0
        L.kg_destroy(h)


def test_calls_before_bind_are_call_order_errors():
    L = B.lib()
    rc, h = _create(I.SHAPES["toy"])
    p, _ = B.make_params()
    tok, conf, stop = ctypes.c_int32(), ctypes.c_float(), ctypes.c_int32()
    prompt = (ctypes.c_int32 * 4)(1, 2, 3, 4)
    assert L.kg_prefill(h, ctypes.byref(p), prompt, 4, ctypes.byref(tok)) == B.KG_ESTATE
    assert b"kg_bind" in L.kg_last_error(h)
    assert L.kg_draft_step(h, ctypes.byref(p), ctypes.byref(tok), ctypes.byref(conf), ctypes.byref(stop)) == B.KG_ESTATE
    buf = (ctypes.c_int32 * 8)()
    n = ctypes.c_int32()
    assert L.kg_verify(h, ctypes.byref(p), buf, ctypes.byref(n)) == B.KG_ESTATE
    assert L.kg_accept(h, ctypes.byref(p), buf, ctypes.byref(n)) == B.KG_ESTATE
    assert L.kg_load_tensor(h, 0, -1, None, 0) == B.KG_ESTATE
    assert L.kg_bind(h, None, 0, None, 0, None, 0, None) == B.KG_EINVAL
    assert L.kg_bind(h, 256, 1, 256, 1, 512, 1, None) == B.KG_ENOSPC          # sizes are checked before any device use
    assert L.kg_bind(h, 257, 1 << 40, 256, 1 << 40, 512, 1 << 40, None) == B.KG_EINVAL   # alignment
    assert L.kg_set_page_order(h, (ctypes.c_int32 * 4)(0, 1, 2, 2), 4) == B.KG_EINVAL
    assert L.kg_set_page_order(h, (ctypes.c_int32 * 4)(3, 1, 2, 0), 4) == B.KG_OK
    assert L.kg_create(None, None) == B.KG_EINVAL
    L.kg_destroy(h)


def test_op_helpers_report_sizes_and_reject_bad_shapes():
    L = B.lib()
    assert L.kg_op_packed_bytes(1, 4096, 4096) == 4096 * 4096 * 2
    assert L.kg_op_packed_bytes(1, 1024, 688) == 1024 * 704 * 2      # K padded to a multiple of 32
    assert L.kg_op_packed_bytes(0, 64, 48) == 64 * 48 * 4
    assert L.kg_op_work_bytes(4096) == 4096 * 32
    assert L.kg_op_pack(1, 256, 17, 64, 256, None) == B.KG_EINVAL
    assert L.kg_op_linear(1, 256, 64, 64, 256, 9, 256, 256, None) == B.KG_EINVAL
    assert L.kg_op_stream_read(None, 1 << 20, 256, None) == B.KG_EINVAL      # NULL source
    assert L.kg_op_stream_read(264, 1 << 20, 256, None) == B.KG_EINVAL       # misaligned source
    assert L.kg_op_stream_read(256, 8, 256, None) == B.KG_EINVAL             # fewer than 16 bytes


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_stats_metrics_match_eq1_eq2_golden_values():
    """kg_stats_cr / kg_stats_ctar on the hand-worked list of tests/golden/metrics_eq1_eq2.txt."""
    S, cr, ct = None, None, {}
    for line in open(os.path.join(ROOT, "tests", "golden", "metrics_eq1_eq2.txt")):
        if line.startswith("#") or not line.strip():
            continue
        p = line.split()
        if p[0] == "S":
            S = [int(v) for v in p[1:]]
        elif p[0] == "CR":
            cr = float(p[1])
        else:
            ct[int(p[1])] = float(p[2])
    st = B.kg_stats()
    st.rounds = len(S)
    for s in S:
        st.s_hist[s] += 1
    assert B.stats_cr(st) == cr
    for w, v in ct.items():
        assert B.stats_ctar(st, w) == v
    with pytest.raises(ValueError):
        B.stats_cr(B.kg_stats())


def test_training_workspace_size_is_host_logic():
    """kg_train_workspace_bytes needs no device: sizes scale with the token capacity, hold the four
    fp32 parameter-sized blocks (master copy, gradient, two AdamW moments), and the capacity is
    limited to 2048 tokens and to max_seq."""
    L = B.lib()
    shape = I.SHAPES["7b"]
    rc, h = _create(shape, max_seq=4100, kv_page_tokens=128)
    assert rc == B.KG_OK
    nb = ctypes.c_size_t()
    sizes = []
    for T in (1, 64, 256):
        assert L.kg_train_workspace_bytes(h, T, ctypes.byref(nb)) == B.KG_OK
        sizes.append(nb.value)
    nparam = 4 * shape.d_model ** 2 + 2 * shape.d_model
    assert sizes[0] >= 4 * nparam * 4 and sizes[0] < sizes[1] < sizes[2] < 4 * nparam * 4 + (1 << 29)
    assert L.kg_train_workspace_bytes(h, 2048, ctypes.byref(nb)) == B.KG_OK and nb.value < 6 * (1 << 30)
    for bad in (0, -3, 2049):
        assert L.kg_train_workspace_bytes(h, bad, ctypes.byref(nb)) == B.KG_EINVAL
    assert L.kg_train_workspace_bytes(h, 8, None) == B.KG_EINVAL
    L.kg_destroy(h)
    rc, h = _create(I.SHAPES["toy"], max_seq=40)
    assert L.kg_train_workspace_bytes(h, 40, ctypes.byref(nb)) == B.KG_OK
    assert L.kg_train_workspace_bytes(h, 41, ctypes.byref(nb)) == B.KG_EINVAL
    # training calls before kg_bind are call-order errors, not crashes
    hp = B.kg_train_params(1e-3, 0.9, 0.999, 1e-8, 0.0)
    toks = (ctypes.c_int32 * 2)(1, 2)
    loss = ctypes.c_double()
    assert L.kg_train_step(h, ctypes.byref(hp), toks, 2, ctypes.byref(loss)) == B.KG_ESTATE
    assert L.kg_train_bind(h, None, 0, 8) == B.KG_ESTATE
    L.kg_destroy(h)


def test_algorithmic_bytes_of_the_benchmark_match_the_shapes():
    """bench.py prices every forward by its algorithmic bytes: weights once plus the cached keys and
    values once.  At the 7B shape these are the hand-computed figures (GB, bf16): a layer 404.75 MB,
    LM head 262.14 MB, adapter 134.22 MB; plain forward 13.215, draft step 1.206, shallow part
    0.8095, verification 12.405; the other adapter architectures change the draft step only."""
    import dataclasses
    import bench
    s = I.SHAPES["7b"]
    fb = bench.forward_bytes(s, 0)
    assert fb["layer"] == (4 * 4096 * 4096 + 3 * 4096 * 11008) * 2 == 404_750_336
    assert fb["head"] == 262_144_000 and fb["adapter"] == 134_217_728
    assert round(fb["plain"] / 1e9, 3) == 13.214 or round(fb["plain"] / 1e9, 3) == 13.215
    assert round(fb["draft"] / 1e9, 3) == 1.206 and round(fb["shallow"] / 1e9, 4) == 0.8095
    assert round(fb["verify"] / 1e9, 3) == 12.405 or round(fb["verify"] / 1e9, 3) == 12.404
    assert fb["plain"] == 32 * fb["layer"] + fb["head"] and fb["verify"] == 30 * fb["layer"] + fb["head"]
    # cached keys and values: 16 KB per token and layer, read once per attention layer of the forward
    ctx = 384
    fk = bench.forward_bytes(s, ctx)
    assert fk["plain"] - fb["plain"] == 32 * 16384 * ctx
    assert fk["draft"] - fb["draft"] == 3 * 16384 * ctx          # two shallow layers and the adapter
    assert fk["verify"] - fb["verify"] == 30 * 16384 * ctx
    d, f, V = s.d_model, s.d_ffn, s.vocab
    draft = {k: bench.forward_bytes(dataclasses.replace(s, adapter=k), 0)["draft"] for k in range(4)}
    assert draft[1] == draft[0]                                   # an own head replaces the shared one byte for byte
    assert draft[2] - draft[0] == 3 * d * f * 2                   # the block's feed-forward
    assert draft[0] - draft[3] == 2 * d * d * 2                   # two maps instead of four


def test_weight_tile_order_is_a_permutation_that_follows_the_waves():
    """The packed bf16 form stores a row tile's KS tiles in the order the projection workgroup
    reads them.  For every KS the map must be a permutation of 0..KS-1 (or tiles would be lost or
    written twice), and wave w, which sums the contiguous k range [w KS / 8, (w + 1) KS / 8), must
    find its i-th tile next to the other waves' i-th tiles: 8 tiles apart from its previous one, with
    the first tile of the one-longer ranges in front."""
    L = B.lib()
    for KS in list(range(1, 130)) + [160, 208, 344, 432, 560, 1000]:
        pos = [L.kg_op_tile_pos(ks, KS) for ks in range(KS)]
        assert sorted(pos) == list(range(KS)), KS
        q, n_long = KS // 8, KS % 8
        for w in range(8):
            ks0, ks1 = (w * KS) // 8, ((w + 1) * KS) // 8
            mine = pos[ks0:ks1]
            regular = mine[1:] if ks1 - ks0 > q else mine
            assert regular == [n_long + w + 8 * j for j in range(q)], (KS, w)
            if ks1 - ks0 > q:
                assert 0 <= mine[0] < n_long, (KS, w)
    assert L.kg_op_tile_pos(-1, 8) == -1 and L.kg_op_tile_pos(8, 8) == -1 and L.kg_op_tile_pos(0, 0) == -1


def test_no_matrix_instruction_sits_in_an_exec_masked_region_without_a_skip_branch(tmp_path):
    """An MFMA ignores the EXEC mask, and the compiler drops the skip branch around a short
    exec-masked region: an `if` on a per-lane copy of a wave-uniform condition that holds nothing
    but an MFMA then runs it also in the waves where the condition is false, on registers they never
    loaded (this once put NaNs into a few logits).  Scan the generated gfx950 code of every kernel:
    walking back from each MFMA through the listing (across labels and across branches on scc / vcc),
    a branch on EXEC or the end of a masked region must come before any instruction that narrows EXEC."""
    import re
    import shutil
    if shutil.which("hipcc") is None:
        pytest.skip("hipcc not available")
    from paper_2404_18911_amd import build as BLD
    asm = open(BLD.device_asm(str(tmp_path / "kangaroo.s"))).read()
    kernels = re.findall(r"^(_Z\w+):", asm, flags=re.M)
    assert any("gemv_bf16_kernel" in k for k in kernels) and any("gemm_prefill" in k for k in kernels)
    n_mfma = 0
    for name in kernels:
        i = asm.index(name + ":")
        j = asm.find(".Lfunc_end", i)
        lines = [l.strip() for l in asm[i:j].split("\n") if l.strip() and not l.strip().startswith(";")]
        for k, line in enumerate(lines):
            if not line.startswith("v_mfma"):
                continue
            n_mfma += 1
            for kk in range(k - 1, -1, -1):
                p = lines[kk]
                assert not p.startswith(("s_and_saveexec", "s_andn2_saveexec", "s_or_saveexec")), (name, k, p)
                # what ends the walk: a branch on EXEC itself (the skip branch of a masked region, or the
                # back edge of a divergent loop), or EXEC being restored / set outright.  Branches on scc
                # or vcc, unconditional branches and labels do not: a region masked before them is
                # still masked after them.
                if p.startswith(("s_cbranch_execz", "s_cbranch_execnz", "s_or_b64 exec", "s_mov_b64 exec", "s_endpgm")):
                    break
    assert n_mfma > 20


def test_the_attention_merge_exchanges_its_partials_with_device_coherent_accesses(tmp_path):
    """The page merge of the decode attention passes partial results between workgroups of one launch
    without a fence: it relies on (1) the partials being stored with agent-scope (sc1, write-through)
    stores, (2) every such store being acknowledged (s_waitcnt vmcnt(0)) before the workgroup bumps the
    head's counter with an atomic add that returns the old value, and (3) the last workgroup reading the
    partials with agent-scope (sc1, cache-bypassing) loads issued after that atomic.  These are properties
    of the generated instructions, not of the source's memory orders, so they are checked on the
    generated gfx950 code of every instantiation."""
    import re
    import shutil
    if shutil.which("hipcc") is None:
        pytest.skip("hipcc not available")
    from paper_2404_18911_amd import build as BLD
    asm = open(BLD.device_asm(str(tmp_path / "kangaroo.s"))).read()
    kernels = [k for k in re.findall(r"^(_Z\w+):", asm, flags=re.M) if "attn_kernel" in k and "pf_attn" not in k]
    assert len(kernels) >= 6
    for name in kernels:
        i = asm.index(name + ":")
        j = asm.find(".Lfunc_end", i)
        lines = [l.strip() for l in asm[i:j].split("\n") if l.strip() and not l.strip().startswith(";")]
        adds = [k for k, l in enumerate(lines) if l.startswith("global_atomic_add")]
        assert len(adds) == 1 and lines[adds[0]].endswith("sc0"), (name, [lines[k] for k in adds])   # returns the old count
        ia = adds[0]
        stores = [k for k in range(ia) if lines[k].startswith("global_store_dword") and lines[k].endswith("sc1")]
        assert len(stores) >= 3, (name, "partials, maxima and sums are stored with sc1")
        waits = [k for k in range(stores[-1] + 1, ia) if lines[k].startswith("s_waitcnt") and "vmcnt(0)" in lines[k]]
        assert waits, (name, "no wait for the stores between the last of them and the counter's atomic")
        # nothing between that wait and the atomic may store partials again
        assert not [k for k in range(waits[-1], ia) if lines[k].startswith("global_store")], name
        loads = [k for k in range(ia, len(lines)) if lines[k].startswith("global_load_dword") and lines[k].endswith("sc1")]
        assert len(loads) >= 3, (name, "the merge reads partials, maxima and sums with sc1")
        # the counter is handed back to zero with the same kind of store
        assert [k for k in range(ia, len(lines)) if lines[k].startswith("global_store_dword") and lines[k].endswith("sc1")], name


def test_profile_reducer_of_bench_reads_rocprof_csv(tmp_path):
    """bench.py --trace-summary on a hand-made rocprofv3 csv tree: per-shape durations, counter means, the
    calibration by the 1 GiB copy, the bytes per projection launch and the per-layer timeline."""
    import subprocess
    import sys
    d = tmp_path / "t" / "vm"
    d.mkdir(parents=True)
    rows = ["Kernel_Name,Grid_Size_X,Grid_Size_Y,Grid_Size_Z,Start_Timestamp,End_Timestamp"]
    t = 1000

    def k(name, gx, dur, gy=1, gap=0):
        nonlocal t
        t += gap
        rows.append(f'"{name}",{gx},{gy},1,{t},{t + dur}')
        t += dur
    for _ in range(2):                                   # two forwards of two layers
        k("void pack_rows_kernel<true>(void const*)", 32768, 4000)
        for _ in range(2):
            k("gemv_bf16_kernel(unsigned int)", 393216, 17000, gap=100)
            k("void attn_kernel<kvhalf_t, 128, true, 1>(AttnArgs)", 16384, 7000, gy=3)
            k("gemv_bf16_kernel(unsigned int)", 131072, 8000)
            k("gemv_bf16_kernel(unsigned int)", 704512, 30000)
            k("gemv_bf16_kernel(unsigned int)", 131072, 16000)
        k("gemv_bf16_kernel(unsigned int)", 1024000, 41000)
        k("head_final_kernel(float const*)", 1024, 5000)
    (d / "1_kernel_trace.csv").write_text("\n".join(rows) + "\n")
    c = tmp_path / "c" / "vm"
    c.mkdir(parents=True)
    crow = ["Kernel_Name,Grid_Size,Counter_Name,Counter_Value"]
    for name, v in (("FETCH_SIZE", 524288.0), ("WRITE_SIZE", 1048576.0)):
        crow.append(f'"__amd_rocclr_copyBuffer",131072,{name},{v}')
    for v in (50000.0, 52000.0):
        crow.append(f'"gemv_bf16_kernel(unsigned int)",393216,FETCH_SIZE,{v}')
        crow.append(f'"gemv_bf16_kernel(unsigned int)",393216,WRITE_SIZE,100.0')
    (c / "2_counter_collection.csv").write_text("\n".join(crow) + "\n")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--trace-summary", f"{tmp_path / 't'},{tmp_path / 'c'}"],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    out = r.stdout
    assert "KERNEL_SOURCE_DIGEST" in out and "2 forwards" in out and "over 2 layers" in out
    assert "one layer (5 kernels + gaps): 78.10 us" in out            # 17 + 7 + 8 + 30 + 16 us and the 0.1 us gap before q,k,v
    # FETCH x 2.0 (the copy reads half of its KiB), WRITE x 1.0: (51000 * 2 + 100) KiB per launch
    line = [l for l in out.splitlines() if l.startswith("TRAFFIC_BYTES_PER_PROJECTION_LAUNCH")][0]
    assert abs(float(line.split()[1]) - (51000 * 2 + 100) * 1024) < 1.0
