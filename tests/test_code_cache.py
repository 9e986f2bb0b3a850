"""Code-object cache of the instantiation step (host only: hipRTC cross-compiles without a GPU)."""
import glob
import os

import pytest

import paper_2006_05664_amd as P


@pytest.fixture()
def mm_op():
    op = P.opevo_op_create(P.OPEVO_MATMUL, (256, 256, 256), P.OPEVO_BF16)
    yield op
    P.opevo_op_destroy(op)
    P.opevo_code_cache_configure(None, 256 << 20)
    P.opevo_code_cache_clear()


CFG_A = [4, 2, 2, 16, 4, 2, 2, 16, 16, 16, 1]
CFG_B = [4, 2, 2, 16, 4, 2, 2, 16, 8, 32, 0]


def _code(op, cfg):
    k, ms = P.opevo_kernel_build(op, P.OPEVO_TILE4, cfg)
    size = P.opevo_kernel_code_size(k)
    P.opevo_kernel_destroy(k)
    return size, ms


def test_second_build_of_a_member_is_a_memory_hit(mm_op):
    P.opevo_code_cache_configure(None, 256 << 20)
    P.opevo_code_cache_clear()
    s0 = P.opevo_code_cache_stats()
    size1, ms1 = _code(mm_op, CFG_A)
    s1 = P.opevo_code_cache_stats()
    assert s1["misses"] == s0["misses"] + 1 and s1["hits"] == s0["hits"]
    assert s1["entries"] == 1 and s1["bytes"] == size1
    size2, ms2 = _code(mm_op, CFG_A)
    s2 = P.opevo_code_cache_stats()
    assert s2["hits"] == s1["hits"] + 1 and s2["misses"] == s1["misses"]
    assert size2 == size1 and ms2 < ms1 / 10
    # another member is another key
    _code(mm_op, CFG_B)
    s3 = P.opevo_code_cache_stats()
    assert s3["misses"] == s2["misses"] + 1 and s3["entries"] == 2


def test_memory_limit_drops_the_oldest_and_zero_switches_off(mm_op):
    P.opevo_code_cache_clear()
    size_a, _ = _code(mm_op, CFG_A)
    P.opevo_code_cache_clear()
    P.opevo_code_cache_configure(None, size_a + 16)       # room for one entry only
    _code(mm_op, CFG_A)
    _code(mm_op, CFG_B)
    s = P.opevo_code_cache_stats()
    assert s["entries"] == 1 and s["bytes"] <= size_a + 16
    before = P.opevo_code_cache_stats()
    _code(mm_op, CFG_B)                                  # the newest stayed
    assert P.opevo_code_cache_stats()["hits"] == before["hits"] + 1
    _code(mm_op, CFG_A)                                  # the oldest went
    assert P.opevo_code_cache_stats()["misses"] == before["misses"] + 1
    P.opevo_code_cache_configure(None, 0)
    assert P.opevo_code_cache_stats()["entries"] == 0
    m = P.opevo_code_cache_stats()["misses"]
    _code(mm_op, CFG_A)
    _code(mm_op, CFG_A)
    assert P.opevo_code_cache_stats()["misses"] == m + 2


def test_directory_survives_clearing_and_damaged_files_are_recompiled(mm_op, tmp_path):
    d = str(tmp_path / "cache")
    P.opevo_code_cache_clear()
    P.opevo_code_cache_configure(d, 256 << 20)
    size1, _ = _code(mm_op, CFG_A)
    files = glob.glob(os.path.join(d, "*.co"))
    assert len(files) == 1 and os.path.getsize(files[0]) > size1
    assert not glob.glob(os.path.join(d, "*.tmp.*"))
    P.opevo_code_cache_clear()                           # what a new process would see
    s0 = P.opevo_code_cache_stats()
    size2, _ = _code(mm_op, CFG_A)
    s1 = P.opevo_code_cache_stats()
    assert size2 == size1 and s1["disk_hits"] == s0["disk_hits"] + 1 and s1["misses"] == s0["misses"]
    # truncate the file: it no longer matches its stated length, so the member compiles again
    # and the file is rewritten whole
    with open(files[0], "r+b") as fh:
        fh.truncate(os.path.getsize(files[0]) // 2)
    P.opevo_code_cache_clear()
    size3, _ = _code(mm_op, CFG_A)
    s2 = P.opevo_code_cache_stats()
    assert size3 == size1 and s2["misses"] == s1["misses"] + 1
    assert os.path.getsize(files[0]) > size1
    # flip a byte of the stored key: the entry is not trusted
    raw = bytearray(open(files[0], "rb").read())
    raw[20] ^= 0xFF
    open(files[0], "wb").write(bytes(raw))
    P.opevo_code_cache_clear()
    _code(mm_op, CFG_A)
    assert P.opevo_code_cache_stats()["misses"] == s2["misses"] + 1


def test_unwritable_directory_is_an_error(mm_op, tmp_path):
    f = tmp_path / "plain_file"
    f.write_text("x")
    with pytest.raises(P.OpevoError):
        P.opevo_code_cache_configure(str(f), -1)
    with pytest.raises(P.OpevoError):
        P.opevo_code_cache_configure(str(tmp_path / "a" / "b" / "c"), -1)   # parent missing
