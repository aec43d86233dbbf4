"""Argument checks of the C-ABI entry points (host logic only: no GPU needed).

Every call here is rejected by the library's own checks before it touches a device: the
pointer values are made-up addresses that are never dereferenced, and each case breaks exactly
one documented precondition of include/bc.h and expects the status the header names for it.
"""

import pytest

from paper_2510_13797_amd import bc

PTR = 0x7F0000100000          # 16-byte aligned, never dereferenced
ODD = PTR + 4                 # 4-byte aligned only


def shape(B=2, Hq=4, Hkv=1, d=64, dtype=bc.BC_F32, scale=0.125):
    return bc.bc_shape(B, Hq, Hkv, d, dtype, scale)


def cache(**kw):
    f = dict(k_slab=PTR, v_slab=PTR, base=PTR, cap=PTR, P=PTR, c=PTR, nb=PTR, w=PTR, err=PTR,
             max_cap=64, order=None, uniform_P=0, uniform_cap=0, rows_per_workgroup=0, plan=0)
    f.update(kw)
    return bc.bc_cache(**f)


# every entry point that takes (shape, cache) first, with otherwise acceptable arguments
def _cache_calls():
    return {
        "bc_cache_init": lambda s, c: bc.bc_cache_init(s, c, PTR, PTR, PTR, 8, None),
        "bc_cache_admit": lambda s, c: bc.bc_cache_admit(s, c, PTR, PTR, PTR, 8, None, PTR, None, None),
        "bc_append_kv": lambda s, c: bc.bc_append_kv(s, c, PTR, PTR, None, bc.BC_ROW_TOKEN, None),
        "bc_decode_attn": lambda s, c: bc.bc_decode_attn(s, c, PTR, PTR, None, PTR, 1 << 30, None),
        "bc_compress_evict": lambda s, c: bc.bc_compress_evict(s, c, PTR, PTR, None, 1, None),
        "bc_decode_step": lambda s, c: bc.bc_decode_step(s, c, PTR, PTR, PTR, PTR, None, None, None, PTR,
                                                         1 << 30, None),
        "bc_beacon_step": lambda s, c: bc.bc_beacon_step(s, c, PTR, PTR, PTR, PTR, None, PTR, 1 << 30, None),
        "bc_decode_step_budget": lambda s, c: bc.bc_decode_step_budget(s, c, PTR, PTR, PTR, PTR, None, None,
                                                                       PTR, PTR, PTR, 1 << 30, None),
        "bc_set_ratio": lambda s, c: bc.bc_set_ratio(s, c, PTR, None, None),
        "bc_sort_by_length": lambda s, c: bc.bc_sort_by_length(s, c, None, PTR, None),
    }


BAD_SHAPES = [
    ("no sequences", dict(B=0)),
    ("no query heads", dict(Hq=0)),
    ("no kv heads", dict(Hkv=0)),
    ("query heads not a multiple of kv heads", dict(Hq=5, Hkv=2)),
    ("group of more than eight query heads", dict(Hq=9, Hkv=1)),
    ("head size neither 64 nor 128", dict(d=96)),
    ("unknown element type", dict(dtype=5)),
]


@pytest.mark.parametrize("why,kw", BAD_SHAPES, ids=[w for w, _ in BAD_SHAPES])
def test_bad_shapes_are_shape_errors_everywhere(why, kw):
    bc.load()
    for name, call in _cache_calls().items():
        assert call(shape(**kw), cache()) == bc.BC_ERR_SHAPE, (name, why)
    assert bc.bc_decode_workspace_bytes(shape(**kw), 64) == 0
    assert bc.bc_prefill_bwd_workspace_bytes(shape(**kw), 64) == 0


@pytest.mark.parametrize("field", ["k_slab", "v_slab", "base", "cap", "P", "c", "nb", "w", "err"])
def test_a_missing_cache_table_is_an_argument_error_everywhere(field):
    bc.load()
    for name, call in _cache_calls().items():
        assert call(shape(), cache(**{field: None})) == bc.BC_ERR_ARG, (name, field)


def test_misaligned_slabs_and_empty_capacity_are_argument_errors():
    bc.load()
    for name, call in _cache_calls().items():
        # the uniform-layout promise: capacity equal to max_cap, prompt not longer than it
        assert call(shape(), cache(uniform_P=16, uniform_cap=32)) == bc.BC_ERR_ARG, name
        assert call(shape(), cache(uniform_P=65, uniform_cap=64)) == bc.BC_ERR_ARG, name
        assert call(shape(), cache(uniform_P=-1)) == bc.BC_ERR_ARG, name
        assert call(shape(), cache(uniform_cap=-1)) == bc.BC_ERR_ARG, name
        assert call(shape(), cache(k_slab=ODD)) == bc.BC_ERR_ARG, name
        assert call(shape(), cache(v_slab=ODD)) == bc.BC_ERR_ARG, name
        assert call(shape(), cache(max_cap=0)) == bc.BC_ERR_ARG, name


def test_decode_entry_points_check_their_own_pointers_and_the_workspace():
    s, c = shape(), cache()
    big = 1 << 30
    need = bc.bc_decode_workspace_bytes(s, 64)
    assert need > 0 and need % 16 == 0
    assert bc.bc_decode_workspace_bytes(s, 0) == 0
    # a larger capacity never needs less workspace
    assert bc.bc_decode_workspace_bytes(s, 65536) >= need
    # attention: query and output
    assert bc.bc_decode_attn(s, c, None, PTR, None, PTR, big, None) == bc.BC_ERR_ARG
    assert bc.bc_decode_attn(s, c, PTR, None, None, PTR, big, None) == bc.BC_ERR_ARG
    assert bc.bc_decode_attn(s, c, ODD, PTR, None, PTR, big, None) == bc.BC_ERR_ARG
    assert bc.bc_decode_attn(s, c, PTR, ODD, None, PTR, big, None) == bc.BC_ERR_ARG
    # the softmax scale: finite and not negative (zero is the uniform-weights special case)
    for bad in (-0.125, float("nan"), float("inf"), -float("inf")):
        assert bc.bc_decode_attn(shape(scale=bad), c, PTR, PTR, None, PTR, big, None) == bc.BC_ERR_ARG
        assert bc.bc_decode_step(shape(scale=bad), c, PTR, PTR, PTR, PTR, None, None, None, PTR, big,
                                 None) == bc.BC_ERR_ARG
    # workspace: missing, misaligned, one byte short
    assert bc.bc_decode_attn(s, c, PTR, PTR, None, None, big, None) == bc.BC_ERR_WORKSPACE
    assert bc.bc_decode_attn(s, c, PTR, PTR, None, ODD, big, None) == bc.BC_ERR_WORKSPACE
    assert bc.bc_decode_attn(s, c, PTR, PTR, None, PTR, 0, None) == bc.BC_ERR_WORKSPACE
    # fused steps: the appended row, and the beacon pair given only by half
    assert bc.bc_decode_step(s, c, None, PTR, PTR, PTR, None, None, None, PTR, big, None) == bc.BC_ERR_ARG
    assert bc.bc_decode_step(s, c, PTR, ODD, PTR, PTR, None, None, None, PTR, big, None) == bc.BC_ERR_ARG
    assert bc.bc_decode_step(s, c, PTR, PTR, PTR, PTR, PTR, None, None, PTR, big, None) == bc.BC_ERR_ARG
    assert bc.bc_decode_step(s, c, PTR, PTR, PTR, PTR, PTR, ODD, None, PTR, big, None) == bc.BC_ERR_ARG
    assert bc.bc_decode_step(s, c, PTR, PTR, PTR, PTR, None, None, None, PTR, 0, None) == bc.BC_ERR_WORKSPACE
    assert bc.bc_beacon_step(s, c, None, PTR, PTR, PTR, None, PTR, big, None) == bc.BC_ERR_ARG
    assert bc.bc_beacon_step(s, c, PTR, PTR, PTR, PTR, None, PTR, 0, None) == bc.BC_ERR_WORKSPACE
    # budget rule: the cap table and the live mask are required
    assert bc.bc_decode_step_budget(s, c, PTR, PTR, PTR, PTR, None, None, None, PTR, PTR, big,
                                    None) == bc.BC_ERR_ARG
    assert bc.bc_decode_step_budget(s, c, PTR, PTR, PTR, PTR, None, None, PTR, None, PTR, big,
                                    None) == bc.BC_ERR_ARG
    assert bc.bc_decode_step_budget(s, c, PTR, PTR, PTR, PTR, None, PTR, PTR, PTR, PTR, big,
                                    None) == bc.BC_ERR_ARG


def test_plan_fields_are_checked_per_call():
    # the plan travels with the call: asking for the bf16 matrix-core kernel on an fp32 cache is a
    # shape error, an unknown plan bit or a negative chunk size an argument error
    s = shape(dtype=bc.BC_F32)
    need = cache(plan=bc.BC_PLAN_NEED_MATRIX_KERNEL)
    assert bc.bc_decode_attn(s, need, PTR, PTR, None, PTR, 1 << 30, None) == bc.BC_ERR_SHAPE
    assert bc.bc_decode_attn(s, cache(plan=1 << 20), PTR, PTR, None, PTR, 1 << 30, None) == bc.BC_ERR_ARG
    assert bc.bc_decode_attn(s, cache(rows_per_workgroup=-1), PTR, PTR, None, PTR, 1 << 30,
                             None) == bc.BC_ERR_ARG
    assert bc.bc_decode_step(s, cache(plan=1 << 20), PTR, PTR, PTR, PTR, None, None, None, PTR, 1 << 30,
                             None) == bc.BC_ERR_ARG
    # a forced chunk size on a large batch may need more workspace than the sizing call promises
    big = shape(B=128, Hq=4, Hkv=1, d=128, dtype=bc.BC_BF16)
    need_ws = bc.bc_decode_workspace_bytes(big, 4096)
    many = cache(max_cap=4096, rows_per_workgroup=256)       # 16 chunks per sequence
    assert bc.bc_decode_attn(big, many, PTR, PTR, None, PTR, need_ws, None) == bc.BC_ERR_WORKSPACE


def test_cache_maintenance_entry_points():
    s, c = shape(), cache()
    assert bc.bc_append_kv(s, c, None, PTR, None, bc.BC_ROW_TOKEN, None) == bc.BC_ERR_ARG
    assert bc.bc_append_kv(s, c, PTR, ODD, None, bc.BC_ROW_TOKEN, None) == bc.BC_ERR_ARG
    assert bc.bc_append_kv(s, c, PTR, PTR, None, 7, None) == bc.BC_ERR_ARG
    # a compression needs either a beacon row or the full-window rule
    assert bc.bc_compress_evict(s, c, None, None, None, 0, None) == bc.BC_ERR_ARG
    assert bc.bc_compress_evict(s, c, PTR, None, None, 1, None) == bc.BC_ERR_ARG
    assert bc.bc_compress_evict(s, c, ODD, PTR, None, 1, None) == bc.BC_ERR_ARG
    assert bc.bc_set_ratio(s, c, None, None, None) == bc.BC_ERR_ARG
    assert bc.bc_cache_init(s, c, PTR, PTR, None, 8, None) == bc.BC_ERR_ARG
    assert bc.bc_cache_init(s, c, PTR, PTR, PTR, -1, None) == bc.BC_ERR_ARG
    assert bc.bc_cache_admit(s, c, PTR, PTR, PTR, 8, None, None, None, None) == bc.BC_ERR_ARG
    assert bc.bc_sort_by_length(s, c, None, None, None) == bc.BC_ERR_ARG
    assert bc.bc_sort_by_length(shape(B=4097), c, None, PTR, None) == bc.BC_ERR_SHAPE
    assert bc.bc_workspace_init(None, 64, None) == bc.BC_ERR_ARG
    assert bc.bc_workspace_init(PTR + 2, 64, None) == bc.BC_ERR_ARG
    assert bc.load().bc_tables_to_host(None, None, None, None, None, None) == bc.BC_ERR_ARG


def test_prefill_entry_points():
    ok = shape(B=1, Hq=4, Hkv=2, d=128, dtype=bc.BC_BF16, scale=0.0884)
    fwd = lambda s, q=PTR, out=PTR, max_rows=64: bc.bc_prefill_attn(s, q, PTR, PTR, PTR, PTR, PTR, max_rows,
                                                                    out, None, None)
    assert fwd(shape(B=1, Hq=4, Hkv=2, d=128, dtype=bc.BC_F32)) == bc.BC_ERR_SHAPE
    assert fwd(shape(B=1, Hq=4, Hkv=2, d=64, dtype=bc.BC_F32)) == bc.BC_ERR_SHAPE
    assert fwd(shape(B=1, Hq=4, Hkv=2, d=64, dtype=bc.BC_BF16), q=None) == bc.BC_ERR_ARG      # (a supported shape)
    assert fwd(ok, q=None) == bc.BC_ERR_ARG
    assert fwd(ok, out=ODD) == bc.BC_ERR_ARG
    assert fwd(ok, max_rows=0) == bc.BC_ERR_ARG
    assert fwd(ok, max_rows=1 << 26) == bc.BC_ERR_ARG
    assert fwd(shape(B=1, Hq=4, Hkv=2, d=128, dtype=bc.BC_BF16, scale=0.0)) == bc.BC_ERR_ARG
    for bad in (float("nan"), float("inf"), -1.0):
        assert fwd(shape(B=1, Hq=4, Hkv=2, d=128, dtype=bc.BC_BF16, scale=bad)) == bc.BC_ERR_ARG

    # the workspace form of the forward: the same checks, plus its workspace
    wsneed = bc.bc_prefill_workspace_bytes(ok, 64)
    assert wsneed == 256 + 64 * 2 * 128 * 2 and bc.bc_prefill_workspace_bytes(ok, 0) == 0
    fws = lambda s=ok, q=PTR, max_rows=64, total=64, ws=PTR, nbytes=1 << 40: bc.bc_prefill_attn_ws(
        s, q, PTR, PTR, PTR, PTR, PTR, max_rows, total, PTR, None, ws, nbytes, None)
    assert fws(s=shape(B=1, Hq=4, Hkv=2, d=128, dtype=bc.BC_F32)) == bc.BC_ERR_SHAPE
    assert fws(q=None) == bc.BC_ERR_ARG
    assert fws(max_rows=65, total=64) == bc.BC_ERR_ARG
    assert fws(ws=None) == bc.BC_ERR_WORKSPACE
    assert fws(ws=ODD) == bc.BC_ERR_WORKSPACE
    assert fws(nbytes=wsneed - 1) == bc.BC_ERR_WORKSPACE

    need = bc.bc_prefill_bwd_workspace_bytes(ok, 64)
    assert need > 0
    assert bc.bc_prefill_bwd_workspace_bytes(ok, 0) == 0
    assert bc.bc_prefill_bwd_workspace_bytes(ok, 128) >= need

    def bwd(s=ok, dq=PTR, lse=PTR, max_rows=64, total=64, ws=PTR, ws_bytes=1 << 40):
        return bc.bc_prefill_attn_bwd(s, PTR, PTR, PTR, PTR, lse, PTR, PTR, PTR, PTR, max_rows, total, dq,
                                      PTR, PTR, ws, ws_bytes, None)
    assert bwd(s=shape(B=1, Hq=4, Hkv=2, d=128, dtype=bc.BC_F32)) == bc.BC_ERR_SHAPE
    ok64 = shape(B=1, Hq=4, Hkv=2, d=64, dtype=bc.BC_BF16, scale=0.125)
    assert bwd(s=ok64, dq=None) == bc.BC_ERR_ARG                                             # (a supported shape)
    assert bc.bc_prefill_bwd_workspace_bytes(ok64, 64) < need                                # partials of D floats per row
    assert bwd(dq=None) == bc.BC_ERR_ARG
    assert bwd(dq=ODD) == bc.BC_ERR_ARG
    assert bwd(lse=None) == bc.BC_ERR_ARG
    assert bwd(max_rows=0) == bc.BC_ERR_ARG
    for bad in (0.0, float("nan"), float("inf"), -1.0):
        assert bwd(s=shape(B=1, Hq=4, Hkv=2, d=128, dtype=bc.BC_BF16, scale=bad)) == bc.BC_ERR_ARG
    assert bwd(max_rows=65, total=64) == bc.BC_ERR_ARG      # a sequence cannot have more rows than the batch
    assert bwd(ws=None) == bc.BC_ERR_WORKSPACE
    assert bwd(ws=ODD) == bc.BC_ERR_WORKSPACE
    assert bwd(ws_bytes=need - 1) == bc.BC_ERR_WORKSPACE


def test_distillation_and_diagnostic_entry_points():
    loss = lambda T=4, V=256, k=10, z=PTR, dt=bc.BC_BF16, out=PTR: bc.bc_topk_kl_loss(
        T, V, k, z, dt, PTR, PTR, out, None, None, None)
    assert loss(k=300) == bc.BC_ERR_SHAPE          # more teacher entries than vocabulary
    assert loss(k=0) == bc.BC_ERR_SHAPE
    assert loss(V=0) == bc.BC_ERR_SHAPE
    assert loss(T=-1) == bc.BC_ERR_SHAPE
    assert loss(T=1 << 31) == bc.BC_ERR_SHAPE
    assert loss(dt=7) == bc.BC_ERR_SHAPE
    assert loss(z=None) == bc.BC_ERR_ARG
    assert loss(out=None) == bc.BC_ERR_ARG
    assert loss(T=0) == bc.BC_OK                   # nothing to do, nothing launched
    grad = lambda lse=PTR, dz=PTR + 4096, z=PTR: bc.bc_topk_kl_loss_bwd(4, 256, 10, z, bc.BC_BF16, PTR, PTR,
                                                                       lse, 1.0, dz, None)
    assert grad(lse=None) == bc.BC_ERR_ARG
    assert grad(dz=None) == bc.BC_ERR_ARG
    assert grad(dz=PTR, z=PTR) == bc.BC_ERR_ARG    # in-place gradients are not supported



def test_measurement_aid_checks_its_arguments():
    assert bc.bc_diag_stream_read(PTR, 1 << 20, 0, 0, PTR, None) == bc.BC_ERR_ARG
    assert bc.bc_diag_stream_read(PTR, 1 << 20, 65537, 0, PTR, None) == bc.BC_ERR_ARG
    assert bc.bc_diag_stream_read(PTR, (1 << 20) + 8, 256, 0, PTR, None) == bc.BC_ERR_ARG
    assert bc.bc_diag_stream_read(PTR, (1 << 20) + 16, 256, 1, PTR, None) == bc.BC_ERR_ARG
    assert bc.bc_diag_stream_read(ODD, 1 << 20, 256, 0, PTR, None) == bc.BC_ERR_ARG
    assert bc.bc_diag_stream_read(None, 1 << 20, 256, 0, PTR, None) == bc.BC_ERR_ARG
    assert bc.bc_diag_stream_read(PTR, 1 << 20, 256, 2, PTR, None) == bc.BC_ERR_ARG


def test_every_status_has_its_own_text():
    texts = [bc.bc_status_str(s) for s in range(0, -7, -1)]
    assert len(set(texts)) == 7 and all(texts)
    assert bc.bc_status_str(-99) not in texts[:1]


def test_noalloc_step_rejects_what_does_not_fit_its_scratch_array():
    # the allocation-free step checks its arguments like bc_decode_step and its plan against the
    # fixed scratch array, before anything is launched or any device is asked for
    s, c = shape(), cache()
    call = lambda s, c, k=PTR: bc.bc_decode_step_noalloc(s, c, k, PTR, PTR, PTR, None, None, None, None)
    assert call(shape(B=0), c) == bc.BC_ERR_SHAPE
    assert call(s, cache(k_slab=None)) == bc.BC_ERR_ARG
    assert call(s, c, k=None) == bc.BC_ERR_ARG
    assert bc.bc_decode_step_noalloc(s, c, PTR, PTR, PTR, PTR, PTR, None, None, None) == bc.BC_ERR_ARG
    # 1024 pairs in 32 forced chunks each: 128 MB of partial results against 4 MiB of scratch
    big = shape(B=128, Hq=64, Hkv=8, d=128, dtype=bc.BC_BF16)
    assert call(big, cache(max_cap=4096, rows_per_workgroup=128)) == bc.BC_ERR_WORKSPACE
    # more counters than the array holds (128 bytes per sequence)
    assert call(shape(B=40000, Hq=1, Hkv=1, d=128, dtype=bc.BC_BF16), cache(max_cap=64)) == bc.BC_ERR_WORKSPACE
