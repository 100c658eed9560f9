"""The C-ABI library loads without a GPU and exports every symbol include/akv.h and include/akw.h declare; host-only entry
points (layout query, argument checks) behave as documented.  No compute call is made here."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def A():
    from paper_2409_16546_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2409_16546_amd import build
        build.build_library(verbose=False)
    return binding


def declared_functions():
    names = set()
    for header in ("akv.h", "akw.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(ak[vw]_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_header_and_binding_name_the_same_entry_points(A):
    names = declared_functions()
    assert names == sorted(A.EXPORTS)
    L = A.lib()
    for n in names:
        assert getattr(L, n) is not None          # dlsym finds every declared symbol
    assert A.akv_version() >= 100


def test_layout_sizes_is_a_host_computation(A):
    sz = A.akv_layout_sizes(8, 32, 32, 128, 4096)
    e = 8 * 32 * 4096 * 128
    assert (sz.k_hi, sz.k_mid, sz.k_lo, sz.v_hi, sz.v_mid, sz.v_lo) == (e, e // 2, e // 2, e, e // 2, e // 2)
    assert sz.k_hi + sz.k_mid + sz.k_lo == 2 * e  # planes hold exactly the fp16 bytes: lossless, no padding
    assert sz.colmax == 8 * 32 * 128 * 2 and sz.lens == 32 and sz.flags == (4 + 8) * 4
    assert sz.workspace >= 8 * 32 * 4096 * 4 and sz.workspace % 256 == 0 and sz.fp16_workspace % 256 == 0


@pytest.mark.parametrize("shape", [(0, 4, 4, 128, 256), (1, 4, 3, 128, 256), (1, 4, 4, 64, 256), (1, 4, 4, 128, 100),
                                   (1, 32, 2, 128, 256), (1, 6, 2, 128, 256)])
def test_bad_shapes_are_refused_with_a_message(A, shape):
    with pytest.raises(A.AkvError) as e:
        A.akv_layout_sizes(*shape)
    assert e.value.status == A.AKV_EINVAL and "bad shape" in str(e.value)


def test_struct_layouts_match_the_header(A):
    # the binding's ctypes structs mirror the C structs field for field
    text = open(os.path.join(ROOT, "include", "akv.h")).read()
    text += open(os.path.join(ROOT, "include", "akw.h")).read()
    for struct, cls in (("akv_shape", A.akv_shape), ("akv_sizes", A.akv_sizes), ("akv_cache", A.akv_cache),
                        ("akv_debug", A.akv_debug), ("akv_stats", A.akv_stats), ("akv_params", A.akv_params),
                        ("akw_weights", A.akw_weights),
                        ("akw_sizes", A.akw_sizes), ("akw_params", A.akw_params)):
        body = re.search(r"typedef struct %s \{(.*?)\} %s;" % (struct, struct), text, flags=re.S).group(1)
        body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
        fields = []
        for decl in body.split(";"):
            decl = decl.strip()
            if not decl:
                continue
            names = re.sub(r"\[\d+\]", "", decl).replace("*", " ").split(",")
            first = names[0].split()[-1]
            fields += [first] + [n.strip() for n in names[1:]]
        assert fields == [f[0] for f in cls._fields_], struct


def test_weight_layout_sizes_and_shape_checks(A):
    sz = A.akw_layout_sizes(4096, 11008)
    e = 4096 * 11008
    assert (sz.hi, sz.mid, sz.lo, sz.rowmax) == (e, e // 2, e // 2, 4096 * 2)
    assert sz.workspace % 256 == 0 and sz.workspace >= (4096 // 512) * 4 * 11008 * 4
    for bad in ((4096, 11000), (4100, 4096), (0, 16), (65536, 32768)):
        with pytest.raises(A.AkvError) as e_:
            A.akw_layout_sizes(*bad)
        assert e_.value.status == A.AKV_EINVAL and "bad shape" in str(e_.value)


def test_misaligned_pointers_are_refused_before_anything_is_launched(A):
    # the addresses are made up: every call below is turned away by the host-side checks, which come first
    L = A.lib()
    planes = {n: 0x10000 * (i + 1) for i, n in enumerate(("k_hi", "k_mid", "k_lo", "v_hi", "v_mid", "v_lo", "colmax",
                                                           "lens", "flags"))}
    shape = A.akv_shape(1, 4, 4, 128, 256)
    good = A.akv_cache(shape, **planes)
    q, out, ws = 0x200000, 0x300000, 0x400000

    def refused(st, word):
        assert st == A.AKV_EINVAL and word in L.akv_last_error().decode()

    refused(L.akv_decode_attention(C.byref(good), q + 2, out, None, ws, 1 << 30, None), "aligned")
    refused(L.akv_decode_attention(C.byref(good), q, out + 4, None, ws, 1 << 30, None), "aligned")
    refused(L.akv_append_decode_attention(C.byref(good), q + 8, q, q, out, None, ws, 1 << 30, None), "aligned")
    for name in ("k_hi", "v_lo", "colmax"):
        bad = A.akv_cache(shape, **{**planes, name: planes[name] + 8})
        refused(L.akv_decode_attention(C.byref(bad), q, out, None, ws, 1 << 30, None), "aligned")
    bad = A.akv_cache(shape, **{**planes, "lens": planes["lens"] + 2})
    refused(L.akv_append(C.byref(bad), q, q, None, 1, None), "aligned")
    refused(L.akv_append(C.byref(good), q + 2, q, None, 1, None), "aligned")
    refused(L.akv_unpack(C.byref(good), q + 2, None, None), "aligned")
    refused(L.akv_fp16_decode_attention(C.byref(shape), q, q + 6, q, q, out, 0.0, 0, 0, ws, 1 << 30, None), "aligned")
    assert L.akv_decode_attention(C.byref(good), q, out, None, ws + 16, 1 << 30, None) == A.AKV_EWORKSPACE
    p = A.akv_params(0.0, 0, 0, -1, 0, 0, None, None, 0, 0x500004)
    refused(L.akv_decode_attention(C.byref(good), q, out, C.byref(p), ws, 1 << 30, None), "stats")


def test_static_scratch_entry_point_refuses_shapes_beyond_its_array(A):
    # host-side check only (made-up addresses): the refusal comes before anything touches the device
    L = A.lib()
    planes = {n: 0x10000 * (i + 1) for i, n in enumerate(("k_hi", "k_mid", "k_lo", "v_hi", "v_mid", "v_lo", "colmax",
                                                           "lens", "flags"))}
    for shape in ((4, 32, 8, 128, 131072), (1024, 16, 16, 128, 256)):   # too many logits; too many control words
        sz = A.akv_layout_sizes(*shape)
        big = A.akv_cache(A.akv_shape(*shape), **planes)
        assert L.akv_decode_attention_static(C.byref(big), 0x200000, 0x300000, None, None) == A.AKV_EWORKSPACE
        msg = L.akv_last_error().decode()
        assert str(A.AKV_STATIC_SCRATCH_BYTES) in msg and "static" in msg
        assert sz.workspace + 65536 > A.AKV_STATIC_SCRATCH_BYTES or shape[0] * shape[2] > 8192
    # the header's constant is the binding's
    text = open(os.path.join(ROOT, "include", "akv.h")).read()
    assert re.search(r"#define AKV_STATIC_SCRATCH_BYTES \((\d+)u << 20\)", text).group(1) == str(A.AKV_STATIC_SCRATCH_BYTES >> 20)


def test_decode_path_query_is_a_host_computation(A):
    # 256 compute units are assumed where no device can be asked
    assert A.akv_decode_path(8, 32, 32, 128, 4096) == 3            # configuration 2: head kernel, logits in LDS
    assert A.akv_decode_path(16, 32, 32, 128, 8192) == 3           # configuration 3: two full rounds of single heads
    assert A.akv_decode_path(8, 32, 8, 128, 32768) == 2            # configuration 4: token-split kernels
    assert A.akv_decode_path(8, 32, 32, 128, 16384) == 2           # too long for the head kernel to pay
    assert A.akv_decode_path(8, 32, 32, 128, 16384, 4096) == 3     # ... unless the caller bounds the lengths
    assert A.akv_decode_path(32, 32, 8, 128, 4096) == 1            # groups of four: 64 KB of logits do not fit the LDS share
    assert A.akv_decode_path(1, 6, 2, 128, 256) == 0               # bad shape


def test_misaligned_weight_arrays_are_refused(A):
    L = A.lib()
    w = A.akw_weights(64, 32, 0x10000, 0x20000, 0x30000, 0x40000)
    x, y, ws = 0x50000, 0x60000, 0x70000
    assert L.akw_gemv(C.byref(w), x + 2, 1, y, None, ws, 1 << 30, None) == A.AKV_EINVAL
    assert L.akw_gemv(C.byref(w), x, 1, y + 4, None, ws, 1 << 30, None) == A.AKV_EINVAL
    assert L.akw_pack(C.byref(w), x + 2, None) == A.AKV_EINVAL
    assert L.akw_unpack(C.byref(A.akw_weights(64, 32, 0x10008, 0x20000, 0x30000, 0x40000)), x, None) == A.AKV_EINVAL
    assert "aligned" in L.akv_last_error().decode()
    assert L.akw_gemv(C.byref(w), x, 1, y, None, ws + 8, 1 << 30, None) == A.AKV_EWORKSPACE
