"""CPU-only checks of the C ABI: the library loads, exports what include/ng.h
declares, sizes and argument validation are right, and the host-side integer
bookkeeping behaves (no kernel is run here)."""
import ctypes as C
import os
import re

import pytest
import torch

from paper_2410_16029_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "ng.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(ng_[a-z_]+)\s*\(", text))
    assert {"ng_init_state", "ng_step", "ng_refresh_projector", "ng_query_sizes", "ng_commit_projector",
            "ng_get_counters", "ng_set_counters", "ng_get_status", "ng_strerror", "ng_destroy"} <= names
    lib = C.CDLL(B.LIB_PATH)
    for name in names:
        assert hasattr(lib, name), name


def test_binding_structs_match_the_compiled_header():
    for which, cls in enumerate((B.ng_matrix_desc, B.ng_hparams, B.ng_matrix_buffers, B.ng_matrix_layout)):
        assert B._lib.ng_struct_size(which) == C.sizeof(cls), cls.__name__
    assert B._lib.ng_struct_size(9) == 0
    # the defaults land in the fields the binding names (a shifted layout would scramble them)
    hp = B.ng_default_hparams()
    assert (hp.refresh_power_iters, hp.refresh_oversample, hp.refresh_sweeps) == (2, 8, 30)
    assert (hp.hist_dtype, hp.fisher_norm, hp.carry_history, hp.proj_dtype, hp.seed) == (B.NG_F32, B.NG_NORM_S, 0, B.NG_F32, 0)


def test_query_sizes_c1_and_bf16_layout():
    hp = B.ng_default_hparams()
    assert (hp.s, hp.grad_dtype, hp.adam_mode) == (4, B.NG_F32, B.NG_ADAM_STANDARD)
    assert abs(hp.lambda_ - 1e-3) < 1e-9 and abs(hp.beta2 - 0.999) < 1e-6
    descs = B.make_descs([(256, 512)], 32)
    sizes, ws = B.ng_query_sizes(descs, hp)
    sz = sizes[0]
    assert sz[B.NG_BUF_P] == 256 * 32 * 4
    assert sz[B.NG_BUF_M] == sz[B.NG_BUF_V] == 32 * 512 * 4
    assert sz[B.NG_BUF_H] == 4 * 32 * 512 * 4
    assert sz[B.NG_BUF_N] == 32 * 512 * 4
    assert sz[B.NG_BUF_AUX] == 0
    assert sz[B.NG_BUF_K] >= 4 * 4 * 8 + 4 * 8 + 4 * 4 and sz[B.NG_BUF_K] % 256 == 0
    assert ws > 0
    # bf16, odd n: rows padded to a multiple of 32, N in octets, bf16 copies of P
    hp.grad_dtype = B.NG_BF16
    hp.s = 16
    descs = B.make_descs([(2048, 5461)], 512)
    sizes, _ = B.ng_query_sizes(descs, hp)
    ldn, stored = 5472, 6144                                # M, V, H: three 2048-column panels, the last one padded
    assert sizes[0][B.NG_BUF_M] == 512 * stored * 4
    assert sizes[0][B.NG_BUF_H] == 16 * 512 * stored * 4
    assert sizes[0][B.NG_BUF_N] == (512 // 8) * ldn * 8 * 2
    hp.hist_dtype = B.NG_BF16                               # opt-in: bf16 history slots
    sizes16, _ = B.ng_query_sizes(descs, hp)
    assert sizes16[0][B.NG_BUF_H] == 16 * 512 * stored * 2
    assert sizes16[0][B.NG_BUF_M] == 512 * stored * 4
    hp.hist_dtype = B.NG_F32
    assert sizes[0][B.NG_BUF_AUX] >= 2 * 2048 * 512 * 2
    hp.proj_dtype = B.NG_BF16                               # opt-in: the projector only as its two bf16 copies
    lowmem, _ = B.ng_query_sizes(descs, hp)
    assert lowmem[0][B.NG_BUF_P] == 0 and lowmem[0][B.NG_BUF_AUX] == sizes[0][B.NG_BUF_AUX]
    hp.carry_history = 1                                    # ... which the history carry-over cannot work from
    with pytest.raises(B.NgError) as e:
        B.ng_query_sizes(descs, hp)
    assert e.value.code == B.NG_ERR_HPARAM
    hp.carry_history = 0
    hp.proj_dtype = B.NG_F32
    # right side: the projector is n x r and the r-space state is r x ldm
    hp.hist_dtype = B.NG_F32
    descs = B.make_descs([(5461, 2048)], 512, sides="auto")
    assert descs[0].side == B.NG_SIDE_RIGHT
    right, _ = B.ng_query_sizes(descs, hp)
    assert right[0][B.NG_BUF_P] == 2048 * 512 * 4
    assert right[0][B.NG_BUF_M] == 512 * stored * 4
    descs = B.make_descs([(2048, 5461)], 512)
    # s = 0 keeps one scratch slot for the projected gradient
    hp.s = 0
    sizes, _ = B.ng_query_sizes(descs, hp)
    assert sizes[0][B.NG_BUF_H] == 512 * stored * 4


@pytest.mark.parametrize("mutate,code", [
    (lambda d, hp: setattr(hp, "lambda_", 0.0), B.NG_ERR_HPARAM),
    (lambda d, hp: setattr(hp, "lambda_", -1.0), B.NG_ERR_HPARAM),
    (lambda d, hp: setattr(hp, "beta1", 1.0), B.NG_ERR_HPARAM),
    (lambda d, hp: setattr(hp, "beta2", -0.1), B.NG_ERR_HPARAM),
    (lambda d, hp: setattr(hp, "eps", 0.0), B.NG_ERR_HPARAM),
    (lambda d, hp: setattr(hp, "s", -1), B.NG_ERR_SHAPE),
    (lambda d, hp: setattr(hp, "s", 65), B.NG_ERR_SHAPE),
    (lambda d, hp: setattr(hp, "grad_dtype", 7), B.NG_ERR_DTYPE),
    (lambda d, hp: setattr(hp, "hist_dtype", 5), B.NG_ERR_DTYPE),
    (lambda d, hp: setattr(hp, "hist_dtype", B.NG_BF16), B.NG_ERR_DTYPE),   # bf16 history needs bf16 gradients
    (lambda d, hp: setattr(hp, "fisher_norm", 2), B.NG_ERR_HPARAM),
    (lambda d, hp: setattr(hp, "proj_dtype", 3), B.NG_ERR_DTYPE),
    (lambda d, hp: setattr(hp, "proj_dtype", B.NG_BF16), B.NG_ERR_HPARAM),   # bf16-only projector needs bf16 gradients
    (lambda d, hp: setattr(hp, "adam_mode", 2), B.NG_ERR_DTYPE),
    (lambda d, hp: setattr(hp, "refresh_sweeps", 0), B.NG_ERR_HPARAM),
    (lambda d, hp: setattr(d[0], "r", 0), B.NG_ERR_SHAPE),
    (lambda d, hp: setattr(d[0], "r", 300), B.NG_ERR_SHAPE),      # r > min(m, n)
    (lambda d, hp: setattr(d[0], "m", 0), B.NG_ERR_SHAPE),
    (lambda d, hp: setattr(d[0], "ld_w", 100), B.NG_ERR_SHAPE),   # ld < n
    (lambda d, hp: setattr(d[0], "ld_g", 511), B.NG_ERR_SHAPE),
    (lambda d, hp: setattr(d[0], "side", 2), B.NG_ERR_INVALID_ARG),
])
def test_argument_validation(mutate, code):
    hp = B.ng_default_hparams()
    descs = B.make_descs([(256, 512)], 32)
    mutate(descs, hp)
    with pytest.raises(B.NgError) as e:
        B.ng_query_sizes(descs, hp)
    assert e.value.code == code
    assert B.ng_strerror(code) != "unknown error code"


def test_null_pointers_rejected():
    hp = B.ng_default_hparams()
    descs = B.make_descs([(256, 512)], 32)
    assert B._lib.ng_query_sizes(None, 1, C.byref(hp), None, None) == B.NG_ERR_INVALID_ARG
    assert B._lib.ng_query_sizes(descs, 0, C.byref(hp), None, None) == B.NG_ERR_INVALID_ARG
    assert B._lib.ng_step(None, None, None, 1e-3, None) == B.NG_ERR_INVALID_ARG
    assert B._lib.ng_get_counters(None, 0, None, None, None, None) == B.NG_ERR_INVALID_ARG
    B._lib.ng_destroy(None)


def _host_only_handle(s=3):
    """A handle over host memory: NG_INIT_HOST_ONLY touches no device and lets nothing launch."""
    return B.LayerSet([(64, 96), (96, 64)], 16, s=s, dtype="f32", device="cpu", host_only=True)


def test_host_bookkeeping_without_device():
    ls = _host_only_handle()
    assert ls.counters(0) == (0, 0, 0, 0)
    g = [torch.zeros(64, 96), torch.zeros(96, 64)]
    w = [torch.zeros(64, 96), torch.zeros(96, 64)]
    # no projector yet
    with pytest.raises(B.NgError) as e:
        ls.step(g, w, 1e-3)
    assert e.value.code == B.NG_ERR_NO_PROJECTOR
    # resume counters, bounds checked
    B.ng_set_counters(ls.st, 1, 41, 2, 3, 5)
    assert ls.counters(1) == (41, 2, 3, 5)
    for bad in [(-1, 0, 0, 0), (0, 3, 0, 0), (0, -1, 0, 0), (0, 0, 4, 0), (0, 0, 0, -1)]:
        with pytest.raises(B.NgError):
            B.ng_set_counters(ls.st, 0, *bad)
    with pytest.raises(B.NgError):
        B.ng_get_counters(ls.st, 2)
    # f32 commit without clearing launches nothing: marks the projector valid
    ls.commit_projector(clear_history=False)
    before = [ls.counters(i) for i in range(2)]
    with pytest.raises(B.NgError) as e:
        ls.step(g, w, 1e-3)             # a host-only handle launches nothing
    assert e.value.code == B.NG_ERR_HIP
    assert [ls.counters(i) for i in range(2)] == before   # a failed call leaves the counters alone
    with pytest.raises(B.NgError) as e:
        ls.refresh(g)
    assert e.value.code == B.NG_ERR_HIP
    with pytest.raises(B.NgError) as e:
        ls.commit_projector(clear_history=True)          # clearing the history would launch
    assert e.value.code == B.NG_ERR_HIP
    assert [ls.counters(i) for i in range(2)] == before
    assert ls.status() == B.NG_ERR_HIP
    lay = B.ng_get_layout(ls.st, 0)
    assert lay.ldn == 96 and lay.slot_elems == 16 * 96 and lay.panel_cols == 96
    ls.close()


def test_wide_bf16_states_are_column_panels_and_the_decoder_undoes_them():
    """M, V and the history slots of a bf16 layer set are stored as 2048-column panels where the padded
    row has 2304 elements or more; everything else stays plain row-major."""
    def layout(shape, **kw):
        ls = B.LayerSet([shape], 8, s=2, device="cpu", host_only=True, **kw)
        lay = B.ng_get_layout(ls.st, 0)
        out = (lay.ldn, lay.panel_cols, lay.slot_elems)
        ls.close()
        return out
    assert layout((64, 5461), dtype="bf16") == (5472, 2048, 8 * 6144)           # the last panel is padded
    assert layout((64, 4096), dtype="bf16") == (4096, 2048, 8 * 4096)
    assert layout((64, 2736), dtype="bf16") == (2752, 2048, 8 * 4096)
    assert layout((64, 2304), dtype="bf16") == (2304, 2048, 8 * 4096)
    assert layout((64, 2272), dtype="bf16") == (2272, 2272, 8 * 2272)          # a sliver of a second panel: one
    assert layout((64, 5461), dtype="f32") == (5472, 5472, 8 * 5472)           # fp32 gradients: row-major
    assert layout((64, 5461), dtype="bf16", carry_history=True) == (5472, 5472, 8 * 5472)
    assert layout((5461, 64), dtype="bf16", sides="auto") == (5472, 2048, 8 * 6144)   # right side: r x ldm
    # sizes count the padded last panel
    hp = B.ng_default_hparams()
    hp.grad_dtype, hp.s = B.NG_BF16, 2
    sizes, _ = B.ng_query_sizes(B.make_descs([(64, 4200)], 8), hp)
    assert sizes[0][B.NG_BUF_M] == sizes[0][B.NG_BUF_V] == 8 * 6144 * 4 and sizes[0][B.NG_BUF_H] == 2 * 8 * 6144 * 4
    assert sizes[0][B.NG_BUF_N] == 1 * 4224 * 8 * 2                            # N is not panelled
    # the binding's decoder: element (row, col) sits at p r pw + row pw + (col - p pw)
    ls = B.LayerSet([(64, 4200)], 8, s=2, dtype="bf16", device="cpu", host_only=True)
    r, ldn, pw, stored = 8, 4224, 2048, 8 * 6144
    flat = torch.arange(stored, dtype=torch.float32)
    ls.buffers[0][B.NG_BUF_M].view(torch.float32)[:stored] = flat
    M = ls.M(0)
    assert M.shape == (r, ldn)
    for row, col in [(0, 0), (3, 2047), (0, 2048), (7, 4095), (0, 4096), (5, 4223)]:
        pnl = col // pw
        assert M[row, col] == pnl * r * pw + row * pw + (col - pnl * pw), (row, col)
    hflat = torch.arange(2 * stored, dtype=torch.float32)
    ls.buffers[0][B.NG_BUF_H].view(torch.float32)[:2 * stored] = hflat
    H = ls.H(0)
    assert H.shape == (2, r, ldn) and H[1, 2, 4100] == stored + 2 * r * pw + 2 * pw + 4
    ls.close()


@pytest.mark.skipif(torch.cuda.is_available(), reason="exercises the no-device error path")
def test_failed_table_upload_returns_an_error_and_no_handle():
    # without a device the upload of the tables fails: the restore flag must not hide that
    for no_clear in (False, True):
        with pytest.raises(B.NgError) as e:
            B.LayerSet([(64, 96)], 16, s=2, dtype="f32", device="cpu", no_clear=no_clear)
        assert e.value.code == B.NG_ERR_HIP


def test_workspace_too_small_and_misaligned():
    hp = B.ng_default_hparams()
    descs = B.make_descs([(64, 96)], 16)
    sizes, ws = B.ng_query_sizes(descs, hp)
    bufs = (B.ng_matrix_buffers * 1)()
    keep = []
    for b in range(B.NG_NBUF):
        t = torch.zeros(max(sizes[0][b], 16) + 256, dtype=torch.uint8)
        keep.append(t)
        bufs[0].buf[b] = (t.data_ptr() + 255) // 256 * 256
    wsbuf = torch.zeros(ws + 512, dtype=torch.uint8)
    base = (wsbuf.data_ptr() + 255) // 256 * 256
    st = C.c_void_p()
    rc = B._lib.ng_init_state(descs, bufs, 1, C.byref(hp), C.c_void_p(base), ws - 1, B.NG_INIT_HOST_ONLY, None,
                              C.byref(st))
    assert rc == B.NG_ERR_WORKSPACE
    rc = B._lib.ng_init_state(descs, bufs, 1, C.byref(hp), C.c_void_p(base + 8), ws, B.NG_INIT_HOST_ONLY, None,
                              C.byref(st))
    assert rc == B.NG_ERR_WORKSPACE
    bufs[0].buf[B.NG_BUF_M] = None
    rc = B._lib.ng_init_state(descs, bufs, 1, C.byref(hp), C.c_void_p(base), ws, B.NG_INIT_HOST_ONLY, None,
                              C.byref(st))
    assert rc == B.NG_ERR_INVALID_ARG


def test_sketch_width_is_trimmed_to_a_multiple_of_32_when_that_keeps_r_columns():
    # l = min(r + p, m, n), then the next lower multiple of 32 if that is still >= r
    cases = [((256, 512), 32, 8, 32),     # 40 -> 32
             ((256, 512), 30, 8, 32),     # 38 -> 32 (>= 30)
             ((256, 512), 33, 8, 41),     # 41 -> 32 would drop a wanted column: kept
             ((256, 512), 4, 8, 12),      # 12 -> 0: kept
             ((256, 512), 64, 32, 96),    # already a multiple
             ((40, 512), 36, 8, 40)]      # clamped to m = 40 first; 32 < 36: kept
    for shape, r, p, want in cases:
        ls = B.LayerSet([shape], r, s=2, dtype="f32", device="cpu", host_only=True, oversample=p)
        assert B.ng_get_layout(ls.st, 0).l == want, (shape, r, p)
        ls.close()


def test_microbench_rejects_bad_arguments_before_any_device_call():
    ms, work = C.c_double(), C.c_double()
    lib = B._lib
    buf = (C.c_char * 64)()
    a = C.addressof(buf)
    a16 = (a + 15) & ~15

    def call(which, pa, pb, nbytes, reps):
        return lib.ng_microbench(which, C.c_void_p(pa), C.c_void_p(pb), nbytes, reps, None, C.byref(ms), C.byref(work))

    assert call(7, a16, a16, 16, 1) == B.NG_ERR_INVALID_ARG            # unknown benchmark
    assert call(B.NG_MB_COPY, a16, a16, 16, 0) == B.NG_ERR_INVALID_ARG  # no repetitions
    assert call(B.NG_MB_COPY, a16, a16, 24, 1) == B.NG_ERR_INVALID_ARG  # not whole 16-byte vectors
    assert call(B.NG_MB_COPY, a16 + 4, a16, 16, 1) == B.NG_ERR_INVALID_ARG   # misaligned source
    assert call(B.NG_MB_COPY, a16, a16 + 4, 16, 1) == B.NG_ERR_INVALID_ARG   # misaligned destination
    assert call(B.NG_MB_READ, 0, a16, 16, 1) == B.NG_ERR_INVALID_ARG    # no source
    assert call(B.NG_MB_MFMA_BF16, 0, 0, 16, 1) == B.NG_ERR_INVALID_ARG  # no sink
    assert call(B.NG_MB_MFMA_BF16, 0, a16, 1 << 25, 1) == B.NG_ERR_INVALID_ARG   # loop count beyond the cap
