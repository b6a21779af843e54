"""CPU-only checks of the C ABI: the library loads, exports every symbol the header
declares, and its host-side functions (byte accounting, canonical sign packing,
device-image round trip, argument errors) agree with the oracle and the paper."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2410_23918_amd as B
from oracle import bitstack_oracle as O
from workloads import synth as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        hdr = open(os.path.join(ROOT, "include", header)).read()
        hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
        names |= set(re.findall(r"\b(bitstack_[a-z0-9_]+)\s*\(", hdr))
    assert {"bitstack_linear", "bitstack_pack_blocks", "bitstack_linear_batched", "bitstack_linear_static",
            "bitstack_set_option", "bitstack_probe_read"} <= names
    L = B.lib()
    for name in sorted(names):
        assert hasattr(L, name), name


def test_block_bytes_matches_eq9_and_oracle():
    for o, i in [(4096, 4096), (1024, 4096), (14336, 4096), (4096, 14336), (28672, 8192), (512, 512)]:
        assert B.block_bytes(o, i, 16) == O.block_bytes(o, i, 16)
    assert B.block_bytes(4096, 4096, 16) == 2359296          # 2.25 MiB, printed in the size table
    assert B.block_bytes(4096, 4096, 8) == 0                 # only k = 16
    assert B.block_bytes(4096, 4000, 16) == 0
    assert B.packed_bytes(4096, 4096, 16, 16, 1) >= 16 * 2359296 + 4096 * 4 + 4096 * 4


def test_pack_signs_from_f32_equals_oracle_including_zeros():
    rng = np.random.default_rng(11)
    R = rng.standard_normal((33, 96)).astype(np.float32)
    R[0, :5] = [0.0, -0.0, 1e-38, -1e-38, -0.0]
    R[rng.random(R.shape) < 0.1] = 0.0
    got = B.pack_signs_from_f32(R)
    assert got.dtype == np.uint32
    assert np.array_equal(got, O.pack_signs(O.sign_pm1(R)))


def test_device_image_round_trip_is_bit_exact():
    rng = W.rng_for(1, 50)
    out, inn, n = 96, 768, 3
    s = W.column_scales(rng, inn)
    S, U, V = W.synthetic_blocks(rng, out, inn, n, 16, s, 0.02)
    sw = np.stack([O.pack_signs(S[i]) for i in range(n)])
    img = B.pack_image_host(sw, U, V, s, max_batch=4)
    assert img.nbytes == B.packed_bytes(out, inn, 16, n, 4)
    for b in range(n):
        sw2, U2, V2 = B.unpack_image_host(img, out, inn, 16, n, 4, b)
        assert np.array_equal(sw2, sw[b])
        assert np.array_equal(U2.view(np.uint16), U[b].view(np.uint16))
        assert np.array_equal(V2.view(np.uint16), V[b].view(np.uint16))
    # each block is one contiguous range of exactly Eq. 9's byte count, and the
    # image stores 1/s in front
    assert np.allclose(img[: inn * 4].view(np.float32), 1.0 / s, rtol=1e-7)
    # changing one sign bit changes exactly one bit of the image
    sw3 = sw.copy(); sw3[1, 40, 7] ^= np.uint32(1 << 13)
    img3 = B.pack_image_host(sw3, U, V, s, max_batch=4)
    diff = np.bitwise_xor(img, img3)
    assert int(np.unpackbits(diff).sum()) == 1
    first = int(np.nonzero(diff)[0][0])
    blk0 = (inn * 4 + 255) // 256 * 256
    assert blk0 + B.block_bytes(out, inn) <= first < blk0 + 2 * B.block_bytes(out, inn)


def test_error_codes_on_the_host():
    L = B.lib()
    rng = W.rng_for(1, 51)
    out, inn, n = 32, 256, 1
    s = W.column_scales(rng, inn)
    S, U, V = W.synthetic_blocks(rng, out, inn, n, 16, s, 0.02)
    sw = np.stack([O.pack_signs(S[0])])
    with pytest.raises(B.BitStackError) as e:
        bad = s.copy(); bad[3] = 0.0
        B.pack_image_host(sw, U, V, bad)
    assert e.value.code == -5
    with pytest.raises(B.BitStackError) as e:
        bad = s.copy(); bad[3] = np.inf
        B.pack_image_host(sw, U, V, bad)
    assert e.value.code == -5
    img = B.pack_image_host(sw, U, V, s)
    with pytest.raises(B.BitStackError) as e:
        B.unpack_image_host(img, out, inn, 16, n, 1, 1)
    assert e.value.code == -3
    # too-small buffer, null pointers, bad shapes, unknown option
    small = np.empty(16, np.uint8)
    p = lambda a: a.ctypes.data_as(C.c_void_p)
    assert L.bitstack_pack_image_host(out, inn, 16, n, 1, p(sw), p(U), p(V), p(s), p(small), 16) == -6
    assert L.bitstack_pack_image_host(out, inn, 16, n, 1, None, p(U), p(V), p(s), p(img), img.nbytes) == -1
    assert L.bitstack_pack_image_host(out, 100, 16, n, 1, p(sw), p(U), p(V), p(s), p(img), img.nbytes) == -2
    assert L.bitstack_linear(None, None, 0, None, None) == -1
    assert L.bitstack_set_option(99, 1) == -8
    assert B.strerror(-5).startswith("scale")
    assert B.strerror(0) == "ok"


def test_bench_sign_packing_matches_oracle():
    """bench.py packs its synthetic sign matrices itself (it may touch the oracle only in its CPU
    baseline leg); the words must be the canonical ones."""
    import importlib
    bench = importlib.import_module("bench")
    from oracle import bitstack_oracle as O
    b = bench.Blocks(96, 512, 3, 3)
    assert np.array_equal(b.sign_words(), O.Stack(b.S, b.U, b.V, b.s).sign_words())


def test_staged_block_equals_its_slot_in_the_whole_image():
    """Dynamic loading moves one block at a time: the staged form of block i must be byte for byte
    what packing the whole stack puts into slot i (block bytes by Eq. 9, then the row maxima)."""
    out, inn, n = 96, 768, 3
    rng = W.rng_for(3, 7)
    s = W.column_scales(rng, inn)
    S, U, V = W.synthetic_blocks(rng, out, inn, n, 16, s, 0.02)
    sw = np.stack([O.pack_signs(S[i]) for i in range(n)])
    img = B.pack_image_host(sw, U, V, s, max_batch=2)
    bb = B.block_bytes(out, inn, 16)
    assert B.block_staging_bytes(out, inn, 16) == (bb + 255) // 256 * 256 + (inn * 2 + 255) // 256 * 256
    off_blocks = (inn * 4 + 255) // 256 * 256
    off_vmax = (off_blocks + n * bb + 255) // 256 * 256
    for i in range(n):
        st = B.stage_block_host(sw[i], U[i], V[i])
        assert np.array_equal(st[:bb], img[off_blocks + i * bb: off_blocks + (i + 1) * bb])
        vm_off = (bb + 255) // 256 * 256
        assert np.array_equal(st[vm_off: vm_off + inn * 2], img[off_vmax + i * inn * 2: off_vmax + (i + 1) * inn * 2])
    with pytest.raises(B.BitStackError):
        B.stage_block_host(sw[0], U[0], V[0], np.empty(16, dtype=np.uint8))


def test_kernel_choice_is_host_logic():
    """bitstack_choose_kernel: one token always takes the decode kernel; the materialising path is
    chosen only with a scratch of at least 1024 rows of the dense weight -- the caller's, or the
    activation scratch inside an image packed for that many tokens -- and a stack the restore
    kernel can hold, and only for prefill-sized batches."""
    import paper_2410_23918_amd as B
    big = 1 << 40
    assert B.choose_kernel(4096, 4096, 16, 1, 1, 16) == B.KERNEL_DECODE
    assert B.choose_kernel(4096, 4096, 16, 2048, 1, 16, big) == B.KERNEL_DECODE
    assert B.choose_kernel(28672, 8192, 16, 2048, 2048, 16, big) == B.KERNEL_MATERIALISE
    # no scratch lent: an image packed for 2048 tokens carries 2048 x in fp16 of activation scratch, which
    # holds 2048 rows of the dense weight at a time; one packed for 1000 tokens has too little
    assert B.choose_kernel(28672, 8192, 16, 2048, 2048, 16, 0) == B.KERNEL_MATERIALISE
    assert B.choose_kernel(28672, 8192, 16, 2048, 512, 16, 0) == B.KERNEL_PANEL
    assert B.choose_kernel(28672, 8192, 16, 1000, 1000, 16, 0) == B.KERNEL_PANEL
    # a scratch for fewer rows than the weight has serves slab by slab, down to 1024 rows; below that it is ignored
    assert B.choose_kernel(28672, 8192, 16, 2048, 2048, 16, B.dense_bytes(28672, 8192) - 1) == B.KERNEL_MATERIALISE
    assert B.choose_kernel(28672, 8192, 16, 2048, 2048, 16, 64 << 20) == B.KERNEL_MATERIALISE
    assert B.choose_kernel(28672, 8192, 16, 1000, 1000, 16, 64 << 20) == B.KERNEL_MATERIALISE
    assert B.choose_kernel(28672, 8192, 16, 1000, 1000, 16, 1024 * 8192 * 2 - 1) == B.KERNEL_PANEL
    assert B.choose_kernel(28672, 8192, 16, 2048, 2048, 16, B.dense_bytes(28672, 8192)) == B.KERNEL_MATERIALISE
    assert B.choose_kernel(28672, 8192, 16, 2048, 128, 16, big) in (B.KERNEL_PANEL, B.KERNEL_MATERIALISE)   # measured equal
    assert B.choose_kernel(28672, 8192, 16, 2048, 128, 16, 0) == B.KERNEL_PANEL
    assert B.choose_kernel(14336, 4096, 32, 2048, 2048, B.restore_max_blocks() + 1, big) == B.KERNEL_PANEL
    assert B.choose_kernel(14336, 4096, 16, 16, 16, 16, big) == B.KERNEL_PANEL      # too few tokens to pay for restoring
    assert B.choose_kernel(4096, 4096, 16, 64, 2, 2, big) in (B.KERNEL_DECODE, B.KERNEL_PANEL)
    assert B.choose_kernel(4096, 4096, 16, 64, 2, 0) == B.KERNEL_AUTO
    # where the measured crossovers lie (Llama-3-8B shapes, 16 blocks): two tokens share a decode
    # launch, eight go to the batch kernels; with a scratch buffer the 4096-row shapes take the
    # materialising path from ~65 tokens on (128-row product tiles fill the chip), the 14336-row
    # shape only from ~700
    assert B.choose_kernel(14336, 4096, 16, 2048, 2, 16, 0) == B.KERNEL_DECODE
    assert B.choose_kernel(14336, 4096, 16, 2048, 8, 16, 0) == B.KERNEL_PANEL
    assert B.choose_kernel(4096, 4096, 16, 2048, 128, 16, big) == B.KERNEL_MATERIALISE
    assert B.choose_kernel(4096, 14336, 16, 2048, 128, 16, big) == B.KERNEL_MATERIALISE
    assert B.choose_kernel(14336, 4096, 16, 2048, 128, 16, big) == B.KERNEL_PANEL
    assert B.choose_kernel(14336, 4096, 16, 2048, 512, 16, big) == B.KERNEL_PANEL
    assert B.choose_kernel(14336, 4096, 16, 2048, 1024, 16, big) == B.KERNEL_MATERIALISE
    # the dense product addresses x with 32-bit byte offsets: a batch beyond that stays with the weight-tile kernel
    assert B.choose_kernel(4096, 8192, 4, 3000, 3000, 4, 0) == B.KERNEL_MATERIALISE
    assert B.choose_kernel(4096, 8192, 4, 300000, 300000, 4, 0) == B.KERNEL_PANEL
    # the restore kernel reaches the loaded blocks through 32-bit offsets: 28 blocks of 36864 x 32768 stay
    # below 4 GiB, 29 do not
    assert 28 * B.block_bytes(36864, 32768) < 2 ** 32 <= 29 * B.block_bytes(36864, 32768)
    assert B.choose_kernel(36864, 32768, 29, 2048, 2048, 28, big) == B.KERNEL_MATERIALISE
    assert B.choose_kernel(36864, 32768, 29, 2048, 2048, 29, big) == B.KERNEL_PANEL
    L = B.lib()
    assert L.bitstack_choose_kernel(4096, 100, 16, 1, 1, 1, 0) == -2
    assert L.bitstack_choose_kernel(4096, 4096, 16, 8, 9, 1, 0) == -3
    assert L.bitstack_choose_kernel(4096, 4096, 16, 8, 1, 17, 0) == -3
    assert B.dense_bytes(4096, 100) == 0


def test_decompose_and_dense_entry_points_check_arguments_before_touching_the_device():
    """Every argument error of bitstack_decompose, bitstack_restore_weight and bitstack_linear_dense
    that does not need a handle is reported before any HIP call (no GPU here)."""
    import ctypes as C
    import paper_2410_23918_amd as B
    L = B.lib()
    vp = C.c_void_p
    out, inn = 64, 256
    nb = L.bitstack_decompose_workspace_bytes(out, inn, 16)
    assert nb >= out * inn * 4 + (out + inn) * 32 * 4 * 2
    assert L.bitstack_decompose_workspace_bytes(out, inn, 8) == 0
    assert L.bitstack_decompose_workspace_bytes(out, 100, 16) == 0
    assert L.bitstack_decompose_workspace_bytes(4096, 4096, 16) > L.bitstack_decompose_workspace_bytes(2048, 4096, 16)
    s = np.ones(inn, dtype=np.float32)
    sp = s.ctypes.data_as(vp)
    fake = vp(0x10000000)          # never dereferenced: every call below fails before any device work
    call = lambda **kw: L.bitstack_decompose(kw.get("W", fake), kw.get("s", sp), kw.get("out", out), kw.get("inn", inn),
                                             kw.get("k", 16), kw.get("n", 1), kw.get("it", 0), fake, fake, fake,
                                             kw.get("ws", fake), kw.get("nb", nb), None)
    assert call(W=None) == -1
    assert call(s=None) == -1
    assert call(ws=None) == -1
    assert call(k=8) == -2
    assert call(inn=100) == -2
    assert call(n=-1) == -3
    assert call(it=-1) == -3
    assert call(it=1001) == -3
    bad = s.copy()
    bad[3] = np.inf
    assert call(s=bad.ctypes.data_as(vp)) == -5
    bad[3] = -1.0
    assert call(s=bad.ctypes.data_as(vp)) == -5
    assert call(ws=vp(0x10000010)) == -4
    assert call(W=vp(0x10000004)) == -4
    assert call(nb=nb - 1) == -6
    assert L.bitstack_restore_weight(None, 1, fake, 1 << 30, None) == -1
    assert L.bitstack_linear_dense(fake, 1, None, fake, fake, 0, None) == -1
    assert L.bitstack_linear_dense(None, 1, None, fake, fake, 0, None) == -1
    assert B.restore_max_blocks() == 29
