"""Host-side checks of libpgmoe that need no GPU: the library loads and exports every symbol
the header declares, arguments are validated before anything is launched, and the host
helpers (weight tiling, unique-expert list) are exact."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2308_12066_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "pgmoe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pgmoe_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = header_functions()
    assert len(names) >= 16
    for n in names:
        assert hasattr(B.lib, n), f"{n} declared in pgmoe.h but not exported"
    assert sorted(B.EXPORTS) == names


def cfg(**kw):
    base = dict(d_model=64, d_ff=128, n_experts=8, top_k=2, n_blocks=3, max_tokens=32, dtype=B.BF16,
                slots_per_gen=0, flags=B.FLAG_HOST_ONLY)
    base.update(kw)
    return B.make_config(**base)


@pytest.mark.parametrize("bad", [dict(dtype=7), dict(d_model=0), dict(d_model=96), dict(d_ff=100), dict(n_experts=0),
                                 dict(n_experts=257), dict(top_k=0), dict(top_k=9), dict(n_blocks=0),
                                 dict(max_tokens=0), dict(slots_per_gen=9), dict(flags=64), dict(d_model=4096),
                                 dict(pregate_distance=4), dict(pregate_distance=-1)])
def test_create_rejects_bad_config(bad):
    with pytest.raises(B.PgmoeError) as ei:
        B.Context(cfg(**bad))
    assert ei.value.code == B.EINVAL and "pgmoe_create" in str(ei.value)
    assert B.expert_bytes(cfg(**bad)) == 0


def test_create_rejects_more_than_the_pull_kernels_can_address():
    """The device-side migration numbers 16-byte units with 32 bits: a slot set of 64 GiB or more
    is refused at creation unless the copy-engine path is chosen."""
    big = dict(d_model=32768, d_ff=65536, dtype=B.F32, n_experts=8, top_k=1, max_tokens=8)     # 16 GiB per expert
    with pytest.raises(B.PgmoeError) as ei:
        B.Context(cfg(**big))
    assert ei.value.code == B.EINVAL and "PGMOE_FLAG_FETCH_MEMCPY" in str(ei.value)
    B.Context(cfg(**big, slots_per_gen=3)).close()
    auto = B.Context(cfg(**dict(big, flags=B.FLAG_HOST_ONLY | B.FLAG_FETCH_AUTO)))       # picks the copy engines at that size
    assert auto.migration_engine == "copy_engine"
    auto.close()
    B.Context(cfg(**dict(big, flags=B.FLAG_HOST_ONLY | B.FLAG_FETCH_MEMCPY))).close()


def test_automatic_choice_of_the_migration_engine():
    """PGMOE_FLAG_FETCH_AUTO: copy engines once a block's migration can reach 256 MiB (slots x expert
    bytes) and no expert cache is configured, the pull kernel otherwise; explicit flags are obeyed."""
    large = dict(d_model=1024, d_ff=4096, n_experts=128, top_k=1, max_tokens=64, n_blocks=12)    # 64 slots x 16.8 MB
    base8 = dict(d_model=768, d_ff=3072, n_experts=8, top_k=1, max_tokens=1, n_blocks=6)         # 1 slot x 9.4 MB
    for kw, flags, want in ((large, B.FLAG_FETCH_AUTO, "copy_engine"), (base8, B.FLAG_FETCH_AUTO, "pull"),
                            (large, 0, "pull"), (base8, B.FLAG_FETCH_MEMCPY, "copy_engine"),
                            (dict(large, cache_slots=8), B.FLAG_FETCH_AUTO, "pull"),
                            (dict(large, slots_per_gen=15), B.FLAG_FETCH_AUTO, "pull"),          # 15 x 16 MiB < 256 MiB
                            (dict(large, slots_per_gen=16), B.FLAG_FETCH_AUTO, "copy_engine")):
        c = B.Context(cfg(**kw, flags=B.FLAG_HOST_ONLY | flags))
        assert c.migration_engine == want, (kw, flags)
        c.close()
    with pytest.raises(B.PgmoeError) as ei:
        B.Context(cfg(flags=B.FLAG_HOST_ONLY | B.FLAG_FETCH_AUTO | B.FLAG_FETCH_MEMCPY))
    assert ei.value.code == B.EINVAL and "exclude" in str(ei.value)


def test_expert_bytes():
    assert B.expert_bytes(cfg(d_model=768, d_ff=3072)) == 9437184
    assert B.expert_bytes(cfg(d_model=1024, d_ff=4096)) == 16777216
    assert B.expert_bytes(cfg(d_model=64, d_ff=256, dtype=B.F32)) == 131072


def test_host_only_context_validates_then_refuses_to_launch():
    c = B.Context(cfg())
    buf = np.zeros(1 << 16, dtype=np.uint8)      # 16-byte aligned host memory standing in for pointers
    p = buf.ctypes.data + (-buf.ctypes.data) % 256
    with pytest.raises(B.PgmoeError) as ei:
        c.pregate_topk(p, p, None, 4, p, p)
    assert ei.value.code == B.ENODEVICE
    with pytest.raises(B.PgmoeError) as ei:
        c.pregate_topk(p, p, None, 33, p, p)      # T > max_tokens
    assert ei.value.code == B.EINVAL and "max_tokens" in str(ei.value)
    with pytest.raises(B.PgmoeError) as ei:
        c.pregate_topk(None, p, None, 4, p, p)
    assert ei.value.code == B.EINVAL and "NULL" in str(ei.value)
    with pytest.raises(B.PgmoeError) as ei:
        c.pregate_topk(p + 2, p, None, 4, p, p)
    assert ei.value.code == B.EINVAL and "aligned" in str(ei.value)
    with pytest.raises(B.PgmoeError) as ei:
        c.permute(p, p, -1, p, p, p)
    assert ei.value.code == B.EINVAL
    with pytest.raises(B.PgmoeError) as ei:
        c.combine(p, p, p, 4, None, None, None)
    assert ei.value.code == B.EINVAL and "both" in str(ei.value)
    with pytest.raises(B.PgmoeError) as ei:
        c.combine(p, p, p, 4, p, p, None)
    assert ei.value.code == B.EINVAL
    with pytest.raises(B.PgmoeError) as ei:
        c.expert_ffn(0, p, p, 8, p, p)
    assert ei.value.code == B.ESTATE                # no store registered
    with pytest.raises(B.PgmoeError) as ei:
        c.expert_ffn(3, p, p, 8, p, p)
    assert ei.value.code == B.EINVAL and "block" in str(ei.value)
    with pytest.raises(B.PgmoeError) as ei:
        c.fetch_experts(0, p, 4, None, None)
    assert ei.value.code == B.ESTATE
    eb = B.expert_bytes(c.cfg)
    with pytest.raises(B.PgmoeError) as ei:
        c.register_host_experts(p, eb - 256, 8 * eb)
    assert ei.value.code == B.EINVAL
    with pytest.raises(B.PgmoeError) as ei:
        c.register_host_experts(p, eb, 7 * eb)
    assert ei.value.code == B.EINVAL
    c.register_resident_experts(p, eb, 8 * eb)
    assert c.fetch_experts(1, p, 4, None, None) == -1      # resident store: nothing to migrate
    with pytest.raises(B.PgmoeError) as ei:
        c.expert_ffn(0, p, p, 65, p, p)             # n_rows > max_tokens*k
    assert ei.value.code == B.EINVAL
    with pytest.raises(B.PgmoeError) as ei:
        c.expert_ffn(0, p, p, 8, p, p)
    assert ei.value.code == B.ENODEVICE
    assert c.workspace_bytes > 0
    c.close()


def test_static_scratch_ffn_validates_and_refuses_what_does_not_fit():
    """pgmoe_expert_ffn_static on a host-only context (nothing can be launched, whatever the
    verdict): argument checks as pgmoe_expert_ffn, and a launch whose partial sums or hidden
    activation exceed the library's static buffer is refused with both sizes in the text."""
    buf = np.zeros(1 << 16, dtype=np.uint8)
    p = buf.ctypes.data + (-buf.ctypes.data) % 256
    # float32: the hidden activation [rows, d_ff] in float32 is the scratch: 4096 x 4096 x 4 = 64 MiB
    big_f32 = B.Context(cfg(dtype=B.F32, d_model=64, d_ff=4096, n_experts=4, top_k=1, max_tokens=4096))
    eb = B.expert_bytes(big_f32.cfg)
    big_f32.register_resident_experts(p, eb, 4 * eb)
    with pytest.raises(B.PgmoeError) as ei:
        big_f32.expert_ffn_static(0, p, p, 4096, p)
    assert ei.value.code == B.EINVAL and str(B.STATIC_SCRATCH_BYTES) in str(ei.value) and str(4096 * 4096 * 4) in str(ei.value)
    with pytest.raises(B.PgmoeError) as ei:
        big_f32.expert_ffn_static(0, p, p, 2048, p)       # 32 MiB: fits exactly, so only the missing device stops it
    assert ei.value.code == B.ENODEVICE
    big_f32.close()
    # bf16, 512 rows per expert (the two tiled GEMMs): float32 partials plus the packed hidden activation
    gemm = B.Context(cfg(d_model=768, d_ff=3072, n_experts=8, top_k=1, max_tokens=4096))
    eb = B.expert_bytes(gemm.cfg)
    gemm.register_resident_experts(p, eb, 8 * eb)
    assert "gemm" in gemm.ffn_kernel_name(4096)
    with pytest.raises(B.PgmoeError) as ei:
        gemm.expert_ffn_static(0, p, p, 4096, p)
    assert ei.value.code == B.EINVAL and "pgmoe_expert_ffn" in str(ei.value)
    # the same argument checks as pgmoe_expert_ffn
    with pytest.raises(B.PgmoeError) as ei:
        gemm.expert_ffn_static(0, p, p, 4097, p)
    assert ei.value.code == B.EINVAL and "n_rows" in str(ei.value)
    with pytest.raises(B.PgmoeError) as ei:
        gemm.expert_ffn_static(1, p, p, 8, p)            # a valid call: only the missing device stops it
    assert ei.value.code == B.ENODEVICE
    with pytest.raises(B.PgmoeError) as ei:
        gemm.expert_ffn_static(3, p, p, 8, p)
    assert ei.value.code == B.EINVAL and "block" in str(ei.value)
    with pytest.raises(B.PgmoeError) as ei:
        gemm.expert_ffn_static(0, None, p, 8, p)
    assert ei.value.code == B.EINVAL and "NULL" in str(ei.value)
    with pytest.raises(B.PgmoeError) as ei:
        gemm.expert_ffn_static(0, p + 2, p, 8, p)
    assert ei.value.code == B.EINVAL and "misaligned" in str(ei.value)
    gemm.close()
    fresh = B.Context(cfg())
    with pytest.raises(B.PgmoeError) as ei:
        fresh.expert_ffn_static(0, p, p, 8, p)
    assert ei.value.code == B.ESTATE                     # no store registered
    fresh.close()


def tiled_position(k, n, K, N, nt_major):
    """The layout rule of pgmoe.h retyped in numpy (vectorised over k, n)."""
    kt, nt = k // 32, n // 16
    tile = np.where(nt_major, nt * (K // 32) + kt, kt * (N // 16) + nt)
    lane = (n % 16) + 16 * ((k % 32) // 8)
    return tile * 512 + lane * 8 + (k % 8)


@pytest.mark.parametrize("d,f", [(64, 128), (128, 64), (192, 320)])
def test_pack_is_the_documented_permutation_and_unpack_inverts_it(d, f):
    c = cfg(d_model=d, d_ff=f)
    g = np.random.default_rng(d + f)
    w1 = g.integers(0, 65536, size=(d, f)).astype(np.uint16)
    w2 = g.integers(0, 65536, size=(f, d)).astype(np.uint16)
    blob = np.zeros(2 * d * f, dtype=np.uint16)
    B.pack_expert(c, w1, w2, blob)
    k, n = np.meshgrid(np.arange(d), np.arange(f), indexing="ij")
    exp1 = np.zeros(d * f, dtype=np.uint16)
    exp1[tiled_position(k, n, d, f, True)] = w1
    k, n = np.meshgrid(np.arange(f), np.arange(d), indexing="ij")
    exp2 = np.zeros(d * f, dtype=np.uint16)
    exp2[tiled_position(k, n, f, d, False)] = w2
    assert np.array_equal(blob[: d * f], exp1) and np.array_equal(blob[d * f:], exp2)
    u1, u2 = np.zeros_like(w1), np.zeros_like(w2)
    B.unpack_expert(c, blob, u1, u2)
    assert np.array_equal(u1, w1) and np.array_equal(u2, w2)


def test_check_streams_validates_before_it_launches():
    c = B.Context(cfg())
    out = ctypes.c_int(0)
    assert B.lib.pgmoe_check_streams(None, None, None, ctypes.byref(out)) == B.EINVAL
    assert B.lib.pgmoe_check_streams(c._h, None, None, None) == B.EINVAL
    with pytest.raises(B.PgmoeError) as ei:
        c.check_streams(None, None)
    assert ei.value.code == B.ENODEVICE
    c.close()


def test_nonmoe_standin_setter_validates_its_argument():
    c = B.Context(cfg())
    c.set_nonmoe_standin(0.0)
    c.set_nonmoe_standin(250.0)
    for bad in (-1.0, 100001.0, float("nan"), float("inf")):
        with pytest.raises(B.PgmoeError) as ei:
            c.set_nonmoe_standin(bad)
        assert ei.value.code == B.EINVAL and "outside" in str(ei.value)
    c.close()


def test_every_accepted_bf16_shape_has_an_expert_kernel():
    """pgmoe_create accepts a bf16 d_model only if expert kernels are built for it, and for every
    accepted shape and row count the launch plan names a kernel that exists."""
    built = (64, 128, 256, 512, 768, 1024, 2048)
    for d in range(64, 2049, 64):
        if d in built:
            continue
        with pytest.raises(B.PgmoeError) as ei:
            B.Context(cfg(d_model=d))
        assert ei.value.code == B.EINVAL and "no bf16 expert kernel" in str(ei.value)
    rows = (1, 2, 5, 16, 17, 40, 64, 100, 191, 192, 255, 700, 3000, 4096, 20000)
    for d in built:
        for f in (64, 192, 256, 320, 1024, 3072, 4096):
            for E in (1, 3, 8, 64, 256):
                ctx = B.Context(cfg(d_model=d, d_ff=f, n_experts=E, top_k=1, max_tokens=20000))
                try:
                    for n in rows:
                        assert ctx.ffn_kernel_name(n) is not None, (d, f, E, n)
                finally:
                    ctx.close()


def test_pack_f32_is_plain_concatenation():
    c = cfg(d_model=6, d_ff=10, dtype=B.F32)
    g = np.random.default_rng(0)
    w1 = g.standard_normal((6, 10)).astype(np.float32)
    w2 = g.standard_normal((10, 6)).astype(np.float32)
    blob = np.zeros(120, dtype=np.float32)
    B.pack_expert(c, w1, w2, blob)
    assert np.array_equal(blob, np.concatenate([w1.ravel(), w2.ravel()]))


def test_unique_experts():
    g = np.random.default_rng(3)
    for n, E in ((0, 4), (1, 1), (16, 64), (4096, 128), (200, 256)):
        idx = g.integers(0, E, size=n).astype(np.int32)
        assert np.array_equal(B.unique_experts(idx, E), np.unique(idx))
    with pytest.raises(B.PgmoeError) as ei:
        B.unique_experts(np.array([0, 5, 2], dtype=np.int32), 5)
    assert ei.value.code == B.EBADINDEX
    with pytest.raises(B.PgmoeError) as ei:
        B.unique_experts(np.array([-1], dtype=np.int32), 5)
    assert ei.value.code == B.EBADINDEX


def test_ffn_kernel_name_follows_the_launch_plan():
    def name(n_rows, **kw):
        ctx = B.Context(cfg(**kw))
        try:
            return ctx.ffn_kernel_name(n_rows)
        finally:
            ctx.close()
    assert name(1, d_model=768, d_ff=3072, n_experts=8, top_k=1, max_tokens=1) == "ffn_decode_kernel"
    assert name(4096, d_model=768, d_ff=3072, n_experts=128, top_k=1, max_tokens=4096) == "ffn_fused_kernel"
    assert name(16, d_model=768, d_ff=3072, n_experts=64, top_k=1, max_tokens=16) == "ffn_fused_kernel"
    assert name(4096, d_model=768, d_ff=3072, n_experts=8, top_k=1, max_tokens=4096) == "ffn_gemm_pack_rows_kernel+ffn_gemm_tile_kernel"   # ~512 rows per expert
    assert name(8, d_model=64, d_ff=256, n_experts=8, top_k=1, dtype=B.F32) == "ffn_f32_hidden_kernel+ffn_f32_out_kernel"
