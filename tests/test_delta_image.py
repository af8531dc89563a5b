"""The delta image (file format and hot-swap staging buffer): host-only checks.  The expected bytes of a small
image are assembled here with struct from the layout the header states, not by calling the library twice."""
import struct

import numpy as np
import pytest
import torch


@pytest.fixture(scope="module")
def bd():
    from paper_2402_10193_amd import binding
    binding.lib()
    return binding


def _round_up(v, a):
    return (v + a - 1) // a * a


def _expected_image(outs, ins, k, packed, alpha):
    n = len(outs)
    alpha0 = 32 + 40 * n
    cursor = _round_up(alpha0 + 4 * n * k, 256)
    begin = cursor
    entries, payload = b"", b""
    for m in range(n):
        pbytes = k * outs[m] * (ins[m] // 32) * 4
        entries += struct.pack("<qqQQQ", outs[m], ins[m], cursor, pbytes, alpha0 + 4 * k * m)
        blob = packed[m].astype("<u4").tobytes()
        assert len(blob) == pbytes
        nxt = _round_up(cursor + pbytes, 256)
        payload += blob + b"\0" * (nxt - cursor - pbytes)
        cursor = nxt
    total = cursor
    alphas = b"".join(np.asarray(a, dtype="<f4").tobytes() for a in alpha)
    head_rest = entries + alphas
    head_rest += b"\0" * (begin - 32 - len(head_rest))
    words = np.frombuffer(payload, dtype="<u8")
    checksum = int(words.sum(dtype=np.uint64)) if words.size else 0
    header = b"BDLTv001" + struct.pack("<IIQQ", n, k, total, checksum)
    return header + head_rest + payload


def _case(rng, outs, ins, k):
    packed = [rng.integers(0, 2**32, size=(k, o, i // 32), dtype=np.uint64).astype(np.uint32) for o, i in zip(outs, ins)]
    alpha = [rng.random(k).astype(np.float32) for _ in outs]
    return packed, alpha


def _build(bd, outs, ins, k, packed, alpha):
    return bd.delta_image_build([torch.from_numpy(p.view(np.int32).copy()) for p in packed],
                                [torch.from_numpy(a.copy()) for a in alpha], outs, ins, k, pinned=False)


@pytest.mark.parametrize("outs,ins,k", [([2, 1], [32, 64], 2), ([3], [96], 1), ([16, 5, 7], [256, 32, 160], 3)])
def test_image_bytes_match_the_stated_layout(bd, outs, ins, k):
    rng = np.random.default_rng(5)
    packed, alpha = _case(rng, outs, ins, k)
    want = _expected_image(outs, ins, k, packed, alpha)
    assert bd.delta_image_bytes(outs, ins, k) == len(want)
    image = _build(bd, outs, ins, k, packed, alpha)
    assert image.numpy().tobytes() == want
    assert bd.delta_image_check(image) == (len(outs), k)
    for m in range(len(outs)):
        o, i, po, ao = bd.delta_image_entry(image, m)
        assert (o, i) == (outs[m], ins[m]) and po % 256 == 0
        got = np.frombuffer(want, dtype="<u4", count=k * o * (i // 32), offset=po).reshape(k, o, i // 32)
        assert np.array_equal(got, packed[m])
        assert np.array_equal(np.frombuffer(want, dtype="<f4", count=k, offset=ao), alpha[m])


def test_image_rejects_corruption(bd):
    rng = np.random.default_rng(6)
    outs, ins, k = [4, 2], [64, 32], 2
    packed, alpha = _case(rng, outs, ins, k)
    image = _build(bd, outs, ins, k, packed, alpha)

    def status_of(img, verify=True):
        with pytest.raises(bd.BitDeltaError) as e:
            bd.delta_image_check(img, verify)
        return e.value.status

    bad = image.clone(); bad[0] = ord("X")
    assert status_of(bad) == 9                                   # magic
    bad = image.clone(); bad[8] = 0
    assert status_of(bad) == 9                                   # no matrices
    bad = image.clone(); bad[12] = 9
    assert status_of(bad) == 9                                   # more planes than the library supports
    assert status_of(image[:-256].clone()) == 9                  # shorter than its header says
    bad = image.clone(); bad[32] = 5                             # out of matrix 0 no longer fits packed_bytes
    assert status_of(bad) == 9
    bad = image.clone(); bad[-1] ^= 1                            # payload bit flip: only the checksum sees it
    assert status_of(bad, True) == 9
    assert bd.delta_image_check(bad, False) == (2, 2)
    assert bd.delta_image_bytes([4], [48], 1) == 0 and bd.delta_image_bytes([4], [32], 0) == 0
    assert bd.delta_image_bytes([], [], 1) == 0


def test_file_round_trip_and_io_errors(bd, tmp_path):
    rng = np.random.default_rng(7)
    outs, ins, k = [8, 4], [128, 32], 1
    packed, alpha = _case(rng, outs, ins, k)
    image = _build(bd, outs, ins, k, packed, alpha)
    path = str(tmp_path / "tenant.bdlt")
    bd.delta_file_write(path, image)
    assert (tmp_path / "tenant.bdlt").read_bytes() == image.numpy().tobytes()      # the file is the image
    back = bd.delta_file_read(path, pinned=False)
    assert torch.equal(back, image)
    with pytest.raises(bd.BitDeltaError) as e:
        bd.delta_file_read(str(tmp_path / "missing.bdlt"), pinned=False)
    assert e.value.status == 10
    (tmp_path / "short.bdlt").write_bytes(image.numpy().tobytes()[:-8])
    with pytest.raises(bd.BitDeltaError) as e:
        bd.delta_file_read(str(tmp_path / "short.bdlt"), pinned=False)
    assert e.value.status == 9
    (tmp_path / "junk.bdlt").write_bytes(b"not a delta image at all, but long enough for a header")
    with pytest.raises(bd.BitDeltaError) as e:
        bd.delta_file_read(str(tmp_path / "junk.bdlt"), pinned=False)
    assert e.value.status == 9
    with pytest.raises(bd.BitDeltaError) as e:
        bd.delta_file_write(str(tmp_path / "no_such_dir" / "x.bdlt"), image)
    assert e.value.status == 10
    # upload / install argument checks need no GPU: they fail before anything is enqueued
    L = bd.lib()
    assert L.bd_delta_upload(image.data_ptr(), image.numel(), 0, 0) == 1
    assert L.bd_delta_upload(image.data_ptr(), image.numel(), 4096 + 16, 0) == 3
    assert L.bd_delta_upload(image.data_ptr(), image.numel() - 1, 4096, 0) == 9
    import ctypes
    vp = ctypes.c_void_p
    assert L.bd_delta_install(image.data_ptr(), image.numel(), 4096, 3, 3, (vp * 2)(8192, 16384), (vp * 2)(4096, 4096), 0) == 4
    assert L.bd_delta_install(image.data_ptr(), image.numel(), 4096, 0, 3, (vp * 2)(8192, None), (vp * 2)(4096, 4096), 0) == 1
    assert L.bd_delta_install(image.data_ptr(), image.numel(), 4096, 0, 3, (vp * 2)(8192, 16384 + 4), (vp * 2)(4096, 4096), 0) == 3
