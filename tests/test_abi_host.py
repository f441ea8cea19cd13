"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function the
header declares, and rejects bad arguments before launching anything."""
import ctypes as C

import pytest

from paper_2601_07568_amd import binding as B
from paper_2601_07568_amd import build, synth


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = build.declared_symbols()
    assert {"dllm_prefill_kv", "dllm_denoise_step", "dllm_unmask", "dllm_refresh_cache"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def cfg_for(ms, **kw):
    d = dict(page_tokens=16, max_pages_per_seq=8, n_pages=8, max_batch=2, max_q=32, max_tokens=128)
    d.update(kw)
    return B.make_config(ms, **d)


def fake_ctx(cfg):
    """A context over fake (never dereferenced) device addresses: creation makes no HIP call."""
    L = B.lib()
    lw = (B.LayerW * max(1, cfg.n_layers))()
    for l in range(cfg.n_layers):
        for name, _ in B.LayerW._fields_:
            setattr(lw[l], name, 0x1000)
    w = B.Weights(0x1000, 0x1000, 0x1000, lw)
    ctx = C.c_void_p()
    ws, kv = L.dllm_workspace_bytes(C.byref(cfg)), L.dllm_kv_pool_bytes(C.byref(cfg))
    rc = L.dllm_create(C.byref(ctx), C.byref(cfg), C.byref(w), 0x10000, kv, 0x20000 * 256, ws)
    return rc, ctx, (lw, w), ws, kv


def test_sizes_and_config_validation():
    L = B.lib()
    cfg = cfg_for(synth.TINY)
    assert L.dllm_workspace_bytes(C.byref(cfg)) > 0
    # pool: layers * 2 * pages * heads * page_tokens * head_dim * 4 bytes
    assert L.dllm_kv_pool_bytes(C.byref(cfg)) == 2 * 2 * 8 * 4 * 16 * 64 * 4
    for bad in (dict(page_tokens=0), dict(max_batch=0), dict(n_pages=0)):
        assert L.dllm_workspace_bytes(C.byref(cfg_for(synth.TINY, **bad))) == 0
    import dataclasses
    for field, val in (("head_dim", 48), ("n_kv_heads", 3), ("mask_id", 4096), ("mask_id", -1)):
        ms = dataclasses.replace(synth.TINY, **{field: val})
        assert L.dllm_workspace_bytes(C.byref(cfg_for(ms))) == 0
        rc, ctx, _, _, _ = fake_ctx(cfg_for(ms))
        assert rc == B.DLLM_ESHAPE and not ctx
    ms = dataclasses.replace(synth.TINY, dtype="bf16", d_ff=692)      # bf16 wants multiples of 8
    assert L.dllm_workspace_bytes(C.byref(cfg_for(ms))) == 0


def test_create_rejects_nulls_and_small_buffers():
    L = B.lib()
    cfg = cfg_for(synth.TINY)
    rc, ctx, keep, ws, kv = fake_ctx(cfg)
    assert rc == B.DLLM_OK and ctx
    L.dllm_destroy(ctx)
    lw, w = keep
    out = C.c_void_p()
    assert L.dllm_create(C.byref(out), C.byref(cfg), C.byref(w), 0x10000, kv - 1, 0x20000 * 256, ws) == B.DLLM_ENOSPACE
    assert L.dllm_create(C.byref(out), C.byref(cfg), C.byref(w), 0x10000, kv, 0x20000 * 256, ws - 1) == B.DLLM_ENOSPACE
    assert L.dllm_create(C.byref(out), C.byref(cfg), C.byref(w), None, kv, 0x20000 * 256, ws) == B.DLLM_EINVAL
    assert L.dllm_create(C.byref(out), C.byref(cfg), C.byref(w), 0x10000, kv, 0x20000 * 256 + 8, ws) == B.DLLM_EINVAL
    lw[1].wo = None
    assert L.dllm_create(C.byref(out), C.byref(cfg), C.byref(w), 0x10000, kv, 0x20000 * 256, ws) == B.DLLM_EINVAL
    assert not out
    assert L.dllm_create(None, C.byref(cfg), C.byref(w), 0x10000, kv, 0x20000 * 256, ws) == B.DLLM_EINVAL


def test_calls_validate_before_launching():
    L = B.lib()
    cfg = cfg_for(synth.TINY)
    rc, ctx, keep, _, _ = fake_ctx(cfg)
    assert rc == B.DLLM_OK
    p = 0x3000
    E, S = B.DLLM_EINVAL, B.DLLM_ESHAPE
    # denoise step
    assert L.dllm_denoise_step(ctx, None, 0, 32, 64, p, p, p, p, p, None) == E
    assert L.dllm_denoise_step(ctx, None, 3, 32, 64, p, p, p, p, p, None) == S          # B > max_batch
    assert L.dllm_denoise_step(ctx, None, 1, 33, 64, p, p, p, p, p, None) == S          # Q > max_q
    assert L.dllm_denoise_step(ctx, None, 1, 32, 97, p, p, p, p, p, None) == S          # beyond the block table
    assert L.dllm_denoise_step(ctx, None, 1, 32, -1, p, p, p, p, p, None) == E
    assert L.dllm_denoise_step(ctx, None, 1, 32, 64, None, p, p, p, p, None) == E
    assert L.dllm_denoise_step(ctx, None, 1, 32, 64, p, p, p, None, p, None) == E
    assert L.dllm_denoise_step(None, None, 1, 32, 64, p, p, p, p, p, None) == E
    assert L.dllm_debug_logits(ctx, None, 1, 32, 64, p, p, p, None) == E
    # the step that allocates nothing: same argument rules, and the context must fit the library's array
    assert L.dllm_denoise_step_static(ctx, None, 0, 32, 64, p, p, p, p, p, None) == E
    assert L.dllm_denoise_step_static(ctx, None, 1, 33, 64, p, p, p, p, p, None) == S
    assert L.dllm_denoise_step_static(ctx, None, 1, 32, 64, p, p, p, p, None, None) == E
    assert L.dllm_denoise_step_static(None, None, 1, 32, 64, p, p, p, p, p, None) == E
    rc_big, big, keep_big, ws_big, _ = fake_ctx(cfg_for(synth.TINY, max_tokens=16384))
    assert rc_big == B.DLLM_OK and ws_big > L.dllm_static_scratch_bytes()
    assert L.dllm_denoise_step_static(big, None, 1, 32, 64, p, p, p, p, p, None) == B.DLLM_ENOSPACE
    L.dllm_destroy(big)
    assert L.dllm_debug_hidden(ctx, None, 1, 32, 64, p, p, p, 3, p) == E                # only 2 layers
    # prefill / refresh
    assert L.dllm_prefill_kv(ctx, None, 1, 129, 129, p, p, None, p) == S                # > max_tokens
    assert L.dllm_prefill_kv(ctx, None, 1, 0, 0, p, p, None, p) == E
    assert L.dllm_prefill_kv(ctx, None, 1, 64, 65, p, p, None, p) == E                  # max_seqlen > total
    assert L.dllm_prefill_kv(ctx, None, 3, 64, 64, p, p, None, p) == S
    assert L.dllm_prefill_kv(ctx, None, 1, 64, 64, None, p, None, p) == E
    assert L.dllm_refresh_cache(ctx, None, 1, 64, 64, p, p, None, p, p, p, None) == E   # outputs need n_commit
    assert L.dllm_refresh_cache(ctx, None, 1, 64, 64, p, p, p, p, p, None, None) == E
    # unmask
    assert L.dllm_unmask(ctx, None, 1, 32, 32, p, p, p, 0.9, -1, None, None) == E       # floor must be >= 0
    assert L.dllm_unmask_entropy(ctx, None, 1, 32, 32, p, p, p, 0.45, -1, None, None) == E
    assert L.dllm_unmask_entropy(ctx, None, 1, 32, 5, p, p, p, 0.45, 1, None, None) == E
    assert L.dllm_unmask_entropy(ctx, None, 1, 32, 32, p, p, None, 0.45, 1, None, None) == E
    assert L.dllm_unmask_entropy(ctx, None, 1, 32, 32, p, p, p, float("nan"), 1, None, None) == E
    assert L.dllm_unmask_entropy(ctx, None, 1, 4096, 2048, p, p, p, 0.45, 1, None, None) == S
    # per-block floors and the block state machine
    assert L.dllm_unmask_blocks(ctx, None, 1, 64, 32, p, p, p, 0.45, 1, None, None, None) == E    # floors are required
    assert L.dllm_unmask_blocks(ctx, None, 1, 64, 48, p, p, p, 0.45, 1, p, None, None) == E
    assert L.dllm_fsm_update(ctx, None, 1, 8, 32, None, p, p, 0.1, 0.95, 1, 0, None, None) == E
    assert L.dllm_fsm_update(ctx, None, 1, 0, 32, p, p, p, 0.1, 0.95, 1, 0, None, None) == E
    assert L.dllm_fsm_update(ctx, None, 1, 8, 32, p, p, p, float("nan"), 0.95, 1, 0, None, None) == E
    assert L.dllm_fsm_update(ctx, None, 1, 8, 32, p, p, p, 0.1, 0.95, -1, 0, None, None) == E
    assert L.dllm_fsm_update(ctx, None, 1, 257, 32, p, p, p, 0.1, 0.95, 1, 0, None, None) == S
    # steps with padding rows, windows of the block state machine
    assert L.dllm_denoise_step_var(ctx, None, 1, 32, 64, p, p, None, p, p, p, None) == E           # q_valid is required
    assert L.dllm_fsm_window(ctx, None, 1, 8, 32, 0, p, p, p, 0, p, p, p, p, p) == E                # W >= 1
    assert L.dllm_fsm_window(ctx, None, 1, 8, 32, 2, p, p, p, -1, p, p, p, p, p) == E               # pad token in the vocabulary
    assert L.dllm_fsm_window(ctx, None, 1, 8, 32, 2, p, p, None, 0, p, p, p, p, p) == E
    assert L.dllm_fsm_scatter(ctx, None, 1, 8, 32, 2, p, p, None, p) == E
    # batch compaction and the step over the live sequences
    assert L.dllm_gather_rows(ctx, None, 2, 4, p, p, p, p, 0) == E                                   # src and dst must differ
    assert L.dllm_gather_rows(ctx, None, 2, 0, p, p, p, p + 64, 0) == E
    assert L.dllm_gather_rows(ctx, None, 2, 4, p, None, p, p + 64, 0) == E
    assert L.dllm_scatter_rows(ctx, None, 0, 4, p, p, p, p + 64) == E
    assert L.dllm_denoise_step_live(ctx, None, 1, 32, 64, p, p, None, None, p, p, p, None) == E      # the live count is required
    assert L.dllm_denoise_step_live(ctx, None, 3, 32, 64, p, p, None, p, p, p, p, None) == S
    # trajectory recording, noisy sequences, early stop
    assert L.dllm_unmask_traced(ctx, None, 1, 32, 32, p, p, p, 2.0, 0, 1, 1, None, None, None) == E   # order is required
    assert L.dllm_noisy_sequence(ctx, None, 1, 32, p, p, p, 8, 1.5, p) == E                         # 0 <= t <= 1
    assert L.dllm_noisy_sequence(ctx, None, 1, 32, p, p, None, 8, 0.5, p) == E
    assert L.dllm_eos_scan(ctx, None, 1, 32, p, -1, p, None, None, None) == E
    assert L.dllm_eos_scan(ctx, None, 1, 32, p, 5, p, None, p, None) == E                            # both or neither
    assert L.dllm_unmask(ctx, None, 1, 32, 5, p, p, p, 0.9, 1, None, None) == E         # Q % block_len
    assert L.dllm_unmask(ctx, None, 1, 32, 32, None, p, p, 0.9, 1, None, None) == E
    assert L.dllm_unmask(ctx, None, 1, 32, 32, p, p, p, float("nan"), 1, None, None) == E
    assert L.dllm_unmask(ctx, None, 1, 4096, 2048, p, p, p, 0.9, 1, None, None) == S
    assert L.dllm_set_kernel_mode(ctx, 7) == E
    assert L.dllm_read_status(ctx, None, None) == E
    assert L.dllm_strerror(B.DLLM_ESHAPE).decode().startswith("unsupported")
    L.dllm_destroy(ctx)
    L.dllm_destroy(None)


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", "/nonexistent/libdllm.so")
    with pytest.raises(RuntimeError):
        B.lib()


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N with N > 1 exits with a message before touching torch or the GPU."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=60)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_host_side_code_under_address_and_undefined_behaviour_sanitizers():
    """The library's host code (argument validation, workspace map, context life cycle, launch geometry up to the
    first launch) compiled with AddressSanitizer + UndefinedBehaviorSanitizer on the host side only and driven by
    csrc/host_check_main.cpp through every entry point, without a GPU: the sanitizers abort on a finding, the
    driver counts wrong return codes."""
    import subprocess
    exe = build.build_host_check()
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "host check: 0 failure(s)" in r.stdout
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr


def test_build_refuses_spills_between_lds_copies():
    """The build's check of the generated code: a kernel that counts its own outstanding memory instructions must not
    spill to scratch between its first and last copy into LDS; spills outside that window and in other kernels pass."""
    from paper_2601_07568_amd import build
    head = "_ZN4dllm9k_attn_dlILi128ELi8ELb1EEEvNS_8AttnArgsE:\n"
    bad = head + " global_load_lds_dwordx4 v[0:1], off\n scratch_store_dword off, v3, off\n global_load_lds_dwordx4 v[2:3], off\n s_endpgm\n"
    with pytest.raises(RuntimeError):
        build._check_counted_loops("kernels_attention.hip", bad)
    ok = head + " scratch_load_dword v3, off, off\n global_load_lds_dwordx4 v[0:1], off\n global_load_lds_dwordx4 v[2:3], off\n" \
                " s_waitcnt vmcnt(0)\n scratch_store_dword off, v3, off\n s_endpgm\n"
    build._check_counted_loops("kernels_attention.hip", ok)
    other = "_ZN4dllm14k_attn_combineILi128EEEvPKfS2_iPtiil:\n global_load_lds_dwordx4 v[0:1], off\n scratch_store_dword off, v3, off\n" \
            " global_load_lds_dwordx4 v[2:3], off\n"
    build._check_counted_loops("kernels_attention.hip", other)
