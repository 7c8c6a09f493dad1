"""CPU-only checks of the boundary: the library loads, exports every declared symbol, and
rejects bad arguments on the host before anything touches a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def nq():
    lib = os.path.join(ROOT, "paper_2506_17870_amd", "libnq.so")
    if not os.path.exists(lib):
        from paper_2506_17870_amd import build
        build.build()
    import paper_2506_17870_amd as nq
    return nq


def declared_functions():
    text = open(os.path.join(ROOT, "include", "nq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(nq_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(nq):
    names = declared_functions()
    assert len(names) >= 24
    lib = ctypes.CDLL(nq.LIB_PATH)
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(nq.EXPORTS) == names
    for name in names:
        assert callable(getattr(nq, name)), f"binding lacks {name}"


def test_version_and_status_strings(nq):
    assert nq.nq_version() >= 1
    assert nq.nq_status_string(nq.NQ_OK) == "ok"
    assert "paged out" in nq.nq_status_string(nq.NQ_ERR_NOT_RESIDENT)


def test_packed_bytes(nq):
    # dense: exactly k bits per element on the padded shape
    assert nq.nq_packed_bytes(512, 512, 6) == 512 * 512 * 6 // 8 == 196608
    assert nq.nq_packed_bytes(512, 512, 2) == 65536
    assert nq.nq_packed_bytes(1, 1, 3) == 32 * 64 * 3 // 8
    assert nq.nq_packed_bytes(33, 65, 5) == 64 * 128 * 5 // 8
    assert nq.nq_packed_bytes(0, 64, 5) == 0
    # the paper's words: 21 three-bit or 12 five-bit fields per 64-bit word (Sec. 3.3.4)
    assert nq.nq_packed_bytes(1, 21, 3, nq.NQ_LAYOUT_PAPER_U64) == 8
    assert nq.nq_packed_bytes(1, 22, 3, nq.NQ_LAYOUT_PAPER_U64) == 16
    assert nq.nq_packed_bytes(2, 12, 5, nq.NQ_LAYOUT_PAPER_U64) == 16
    assert nq.nq_packed_bytes(4, 4, 0) == 0 and nq.nq_packed_bytes(4, 4, 8) == 0
    assert nq.nq_packed_bytes(-1, 4, 3) == 0 and nq.nq_packed_bytes(4, 4, 3, 7) == 0


def test_host_side_argument_checks(nq):
    # all of these return before any HIP call: fake non-null addresses are never dereferenced
    a = 0x1000
    with pytest.raises(nq.NQError) as e:
        nq.nq_decompose(a, 4, 4, nq.make_cfg(7, 2), a, a, stream=0)
    assert e.value.status == nq.NQ_ERR_UNSUPPORTED
    for n, l in [(8, 0), (8, 7), (6, 5), (6, 0)]:
        with pytest.raises(nq.NQError) as e:
            nq.nq_decompose_pack(a, 4, 4, nq.make_cfg(n, l), a, a, stream=0)
        assert e.value.status == nq.NQ_ERR_UNSUPPORTED
    with pytest.raises(nq.NQError) as e:
        nq.nq_decompose_pack(a, 4, 4, nq.make_cfg(8, 2, 7), a, a, stream=0)     # no such lower-bit format
    assert e.value.status == nq.NQ_ERR_INVALID_ARG
    # the compensated format is accepted: an empty tensor is a no-op, its page has l + 1 bits per element
    nq.nq_decompose_pack(a, 0, 16, nq.make_cfg(8, 2, nq.NQ_LOW_SIGNED_L1), a, a, stream=0)
    assert nq.nq_packed_bytes(64, 128, 3) == 64 * 128 * 3 // 8
    with pytest.raises(nq.NQError) as e:
        nq.nq_decompose_pack(a, 4, nq.NQ_MAX_K + 1, nq.make_cfg(8, 2), a, a, stream=0)
    assert e.value.status == nq.NQ_ERR_SHAPE
    with pytest.raises(nq.NQError) as e:
        nq.nq_decompose_pack(a, 4, 4, nq.make_cfg(8, 2), a + 4, a, stream=0)
    assert e.value.status == nq.NQ_ERR_ALIGN
    with pytest.raises(nq.NQError) as e:
        nq.nq_decompose_pack(None, 4, 4, nq.make_cfg(8, 2), a, a, stream=0)
    assert e.value.status == nq.NQ_ERR_INVALID_ARG
    with pytest.raises(nq.NQError) as e:
        nq.nq_pack(a, None, 4, 4, nq.make_cfg(8, 2), None, a, stream=0)
    assert e.value.status == nq.NQ_ERR_INVALID_ARG
    # the quantiser: width, pointers, layout, sizes
    with pytest.raises(nq.NQError) as e:
        nq.nq_quantize(a, 4, 4, 9, a, a, stream=0)
    assert e.value.status == nq.NQ_ERR_INVALID_ARG
    with pytest.raises(nq.NQError) as e:
        nq.nq_quantize(a, 4, 4, 8, None, a, stream=0)
    assert e.value.status == nq.NQ_ERR_INVALID_ARG
    with pytest.raises(nq.NQError) as e:
        nq.nq_quantize(a, 4, nq.NQ_MAX_K + 1, 8, a, a, stream=0)
    assert e.value.status == nq.NQ_ERR_SHAPE
    nq.nq_quantize(a, 0, 16, 8, a, a, stream=0)
    # the per-tensor form: width, pointers, alignment (all refused before anything is launched)
    with pytest.raises(nq.NQError) as e:
        nq.nq_quantize_tensor(a, 10, 9, a, a, stream=0)
    assert e.value.status == nq.NQ_ERR_INVALID_ARG
    with pytest.raises(nq.NQError) as e:
        nq.nq_quantize_tensor(a, 10, 8, None, a, stream=0)
    assert e.value.status == nq.NQ_ERR_INVALID_ARG
    with pytest.raises(nq.NQError) as e:
        nq.nq_quantize_tensor(a, 10, 8, a, None, stream=0)
    assert e.value.status == nq.NQ_ERR_INVALID_ARG
    with pytest.raises(nq.NQError) as e:
        nq.nq_quantize_tensor(a + 2, 10, 8, a, a, stream=0)
    assert e.value.status == nq.NQ_ERR_ALIGN
    with pytest.raises(nq.NQError) as e:
        nq.nq_tensor_scale(a, -1, 8, a, stream=0)
    assert e.value.status == nq.NQ_ERR_INVALID_ARG
    with pytest.raises(nq.NQError) as e:
        nq.nq_quantize_decompose_pack(a, 4, 4, nq.make_cfg(8, 2, layout=nq.NQ_LAYOUT_PAPER_U64), a, a, a, stream=0)
    assert e.value.status == nq.NQ_ERR_UNSUPPORTED
    with pytest.raises(nq.NQError) as e:
        nq.nq_quantize_decompose_pack(a, 4, 4, nq.make_cfg(8, 2), None, a, a, stream=0)
    assert e.value.status == nq.NQ_ERR_INVALID_ARG
    with pytest.raises(nq.NQError) as e:
        nq.nq_quantize_decompose_pack(a, 4, 4, nq.make_cfg(8, 2), a, a + 8, a, stream=0)
    assert e.value.status == nq.NQ_ERR_ALIGN
    nq.nq_quantize_decompose_pack(a, 0, 16, nq.make_cfg(6, 2), a, a, a, stream=0)
    # the batched form: the same checks per job, dense layout only, an empty batch is a no-op
    nq.nq_decompose_pack_batch([], nq.make_cfg(8, 2), stream=0)
    nq.nq_decompose_pack_batch([(a, 0, 16, a, a)], nq.make_cfg(8, 2), stream=0)
    with pytest.raises(nq.NQError) as e:
        nq.nq_decompose_pack_batch([(a, 4, 4, a, a), (a, 4, 4, a + 4, a)], nq.make_cfg(8, 2), stream=0)
    assert e.value.status == nq.NQ_ERR_ALIGN
    with pytest.raises(nq.NQError) as e:
        nq.nq_decompose_pack_batch([(a, 4, 4, a, None)], nq.make_cfg(8, 2), stream=0)
    assert e.value.status == nq.NQ_ERR_INVALID_ARG
    with pytest.raises(nq.NQError) as e:
        nq.nq_decompose_pack_batch([(a, 4, 4, a, a)], nq.make_cfg(8, 2, layout=nq.NQ_LAYOUT_PAPER_U64), stream=0)
    assert e.value.status == nq.NQ_ERR_UNSUPPORTED
    # empty tensors are a no-op
    nq.nq_decompose(None, 0, 16, nq.make_cfg(8, 2), None, None, stream=0)
    nq.nq_decompose_pack(a, 0, 16, nq.make_cfg(8, 2), a, a, stream=0)


def test_gemm_argument_checks_without_gpu(nq):
    a = 0x1000
    cfg = nq.make_cfg(8, 2)
    w = nq.nq_weight(cfg, 64, 64, a, 64 * 64 * 6 // 8, a, 64 * 64 * 2 // 8, a, a, 0, 0, None, None, 0, 0)
    epi = nq.make_epilogue()
    # full-bit while the lower-bit page is paged out: an error, never a silent downgrade
    with pytest.raises(nq.NQError) as e:
        nq.nq_gemm_full(a, 8, w, epi, a, stream=0)
    assert e.value.status == nq.NQ_ERR_NOT_RESIDENT
    w.high_bytes = 16
    with pytest.raises(nq.NQError) as e:
        nq.nq_gemm_part(a, 8, w, epi, a, stream=0)
    assert e.value.status == nq.NQ_ERR_RANGE
    w.high_bytes = 64 * 64 * 6 // 8
    w.cfg.layout = nq.NQ_LAYOUT_PAPER_U64
    # the paper's word pages: 7 words of ten 6-bit fields per row, more bytes than the dense page
    with pytest.raises(nq.NQError) as e:
        nq.nq_gemm_part(a, 8, w, epi, a, stream=0)
    assert e.value.status == nq.NQ_ERR_RANGE
    w.high_bytes = 64 * 7 * 8
    with pytest.raises(nq.NQError) as e:
        nq.nq_gemm_part(a + 2, 8, w, epi, a, stream=0)      # activations off a dword boundary
    assert e.value.status == nq.NQ_ERR_ALIGN
    with pytest.raises(nq.NQError) as e:                    # a convolution's input off a dword boundary
        nq.nq_conv_part(a + 2, nq.nq_conv_shape(1, 8, 8, 16, 64, 2, 2, 1, 0), w, epi, a, stream=0)
    assert e.value.status == nq.NQ_ERR_ALIGN
    with pytest.raises(nq.NQError) as e:                    # grouped convolutions read the dense pages only
        nq.nq_gconv_part(a, nq.nq_conv_shape(1, 8, 8, 64, 64, 4, 4, 1, 0), 16, w, epi, a, stream=0)
    assert e.value.status == nq.NQ_ERR_UNSUPPORTED
    w.high_bytes = 64 * 64 * 6 // 8
    w.cfg.layout = nq.NQ_LAYOUT_DENSE
    nq.nq_gemm_part(a, 0, w, epi, a, stream=0)          # M == 0: nothing to do
    shape = nq.nq_conv_shape(1, 8, 8, 16, 64, 3, 3, 1, 1)  # K would be 144, the descriptor says 64
    with pytest.raises(nq.NQError) as e:
        nq.nq_conv_part(a, shape, w, epi, a, stream=0)
    assert e.value.status == nq.NQ_ERR_SHAPE
    # grouped convolution: shape against the descriptor, group size, channel multiple, alignment
    wd = nq.nq_weight(cfg, 64, 9, a, 64 * 64 * 6 // 8, a, 64 * 64 * 2 // 8, a, a, 0, 0, None, None, 0, 0)
    dw = nq.nq_conv_shape(1, 8, 8, 64, 64, 3, 3, 1, 1)
    with pytest.raises(nq.NQError) as e:
        nq.nq_gconv_part(a, dw, 16, wd, epi, a, stream=0)        # groups of 4: K would be 36
    assert e.value.status == nq.NQ_ERR_SHAPE
    with pytest.raises(nq.NQError) as e:
        nq.nq_gconv_part(a, dw, 7, wd, epi, a, stream=0)         # 7 does not divide 64
    assert e.value.status == nq.NQ_ERR_SHAPE
    with pytest.raises(nq.NQError) as e:
        nq.nq_gconv_full(a, dw, 64, wd, epi, a, stream=0)        # lower-bit page not resident
    assert e.value.status == nq.NQ_ERR_NOT_RESIDENT
    with pytest.raises(nq.NQError) as e:
        nq.nq_gconv_part(a, nq.nq_conv_shape(1, 8, 8, 64, 32, 3, 3, 1, 1), 32, wd, epi, a, stream=0)   # the descriptor has 64 rows, not 32
    assert e.value.status == nq.NQ_ERR_SHAPE
    nq.nq_gconv_part(a, nq.nq_conv_shape(0, 8, 8, 64, 64, 3, 3, 1, 1), 64, wd, epi, a, stream=0)      # empty batch
    with pytest.raises(nq.NQError) as e:
        nq.nq_page_in_low(w, 0)                        # nq_weight_init was never called
    assert e.value.status == nq.NQ_ERR_INVALID_ARG
    with pytest.raises(nq.NQError) as e:
        nq.nq_maxpool_i8(a, 1, 4, 4, 8, 3, 2, 3, a, stream=0)
    assert e.value.status == nq.NQ_ERR_SHAPE


def test_batch_paging_argument_checks_without_gpu(nq):
    # descriptors that never went through nq_weight_init_group have no events: rejected on the host
    a = 0x1000
    cfg = nq.make_cfg(8, 2)
    ws = [nq.nq_weight(cfg, 64, 64, a, 64 * 64 * 6 // 8, a, 64 * 64 * 2 // 8, a, a, 0, 0, None, None, 0, 0)
          for _ in range(3)]
    with pytest.raises(nq.NQError) as e:
        nq.nq_page_out_low_batch(ws, 0)
    assert e.value.status == nq.NQ_ERR_INVALID_ARG
    with pytest.raises(nq.NQError) as e:
        nq.nq_page_in_low_batch(ws, 0)
    assert e.value.status == nq.NQ_ERR_INVALID_ARG
    with pytest.raises(nq.NQError) as e:
        nq.nq_page_in_low_batch([], 0)
    assert e.value.status == nq.NQ_ERR_INVALID_ARG
    with pytest.raises(nq.NQError) as e:
        nq.nq_weight_init_group([])
    assert e.value.status == nq.NQ_ERR_INVALID_ARG
    # the first descriptor of a group is checked like a single one: unsupported nesting, short page
    bad = nq.nq_weight(nq.make_cfg(8, 7), 64, 64, a, 64 * 64, a, 64 * 64, a, a, 0, 0, None, None, 0, 0)
    with pytest.raises(nq.NQError) as e:
        nq.nq_weight_init_group([bad])
    assert e.value.status == nq.NQ_ERR_UNSUPPORTED
    short = nq.nq_weight(cfg, 64, 64, a, 16, a, 64 * 64 * 2 // 8, a, a, 0, 0, None, None, 0, 0)
    with pytest.raises(nq.NQError) as e:
        nq.nq_weight_init_group([short])
    assert e.value.status == nq.NQ_ERR_RANGE


def test_group_members_switch_through_the_batch_calls_only(nq):
    # members of a group share their events; the single-page calls on one of them are refused on the host
    a = 0x1000
    cfg = nq.make_cfg(8, 2)
    member = nq.nq_weight(cfg, 64, 64, a, 64 * 64 * 6 // 8, a, 64 * 64 * 2 // 8, a, a)
    member.low_event, member.free_event = 0x10, 0x20     # never dereferenced: the check comes first
    member.events_borrowed = 1
    head = nq.nq_weight(cfg, 64, 64, a, 64 * 64 * 6 // 8, a, 64 * 64 * 2 // 8, a, a)
    head.low_event, head.free_event = 0x10, 0x20
    head.group_head = 1
    for w in (member, head):
        with pytest.raises(nq.NQError) as e:
            nq.nq_page_in_low(w, 0)
        assert e.value.status == nq.NQ_ERR_INVALID_ARG
        with pytest.raises(nq.NQError) as e:
            nq.nq_page_out_low(w, 0)
        assert e.value.status == nq.NQ_ERR_INVALID_ARG
        assert w.low_resident == 0 and w.free_event_armed == 0
    member.low_event = member.free_event = None            # so that nothing tries to destroy the fake handles
    head.low_event = head.free_event = None


def test_tuning_setter_argument_checks(nq):
    for key in (nq.NQ_TUNE_KERNEL, nq.NQ_TUNE_BIG_TM, nq.NQ_TUNE_GC_UNITS, nq.NQ_TUNE_STAT_ROWS):
        nq.nq_set_tuning(key, 3)
        nq.nq_set_tuning(key, 0)
    for key, value in ((-1, 0), (4, 0), (0, -1)):
        with pytest.raises(nq.NQError) as e:
            nq.nq_set_tuning(key, value)
        assert e.value.status == nq.NQ_ERR_INVALID_ARG
