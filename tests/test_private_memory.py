"""Device memory behind the caller's back: the private (stack / register spill) segment of every
kernel in the built library, read from the code objects' metadata, against what the plan reports.

Paper section 4.4: a memory limit holds only if everything that is live is counted.  The
workspace is the caller's; what a kernel spills to private memory is provided by the HIP
runtime for every resident wave.  Every search kernel has none, except the low-d bf16 filter
kernel, whose figure the plan carries (private_bytes) and counts against the limit."""
import os
import re
import struct
import subprocess

import pytest

import paper_2206_14148_amd as K

READELF = "/opt/rocm/llvm/bin/llvm-readelf"


def kernel_private_sizes():
    data = open(K.library_path(), "rb").read()
    out = {}
    at = 0
    magic = b"__CLANG_OFFLOAD_BUNDLE__"
    while True:
        i = data.find(magic, at)
        if i < 0:
            break
        at = i + len(magic)
        (count,) = struct.unpack_from("<Q", data, i + 24)
        off = i + 32
        for _ in range(count):
            o, size, tlen = struct.unpack_from("<QQQ", data, off)
            off += 24
            triple = data[off:off + tlen].decode()
            off += tlen
            if "gfx950" not in triple or size == 0:
                continue
            path = "/tmp/_knn_code_object.elf"
            with open(path, "wb") as f:
                f.write(data[i + o:i + o + size])
            notes = subprocess.run([READELF, "--notes", path], capture_output=True, text=True, check=True).stdout
            os.remove(path)
            for block in notes.split("  - .agpr_count")[1:]:
                name = re.search(r"\.name:\s+(\S+)", block)
                priv = re.search(r"\.private_segment_fixed_size:\s+(\d+)", block)
                if name and priv:
                    out[name.group(1)] = int(priv.group(1))
    return out


@pytest.mark.skipif(not os.path.exists(READELF), reason="llvm-readelf not available")
def test_search_kernels_use_no_private_memory_except_where_the_plan_says_so():
    K.load()
    sizes = kernel_private_sizes()
    search = {n: v for n, v in sizes.items() if "knn_" in n}  # every kernel of the kNN paths
    assert len(search) > 60, sorted(sizes)[:5]
    for family in ("knn_wide_kernel", "knn_packed_kernel", "knn_split_kernel", "knn_seed_kernel", "knn_pack_block_kernel",
                   "knn_merge_refine_kernel", "knn_row_norms_kernel", "knn_lowd_kernel", "knn_l1_kernel"):
        assert any(family in n for n in search), family
    for name, size in search.items():
        if "knn_lowd_bf16_kernel" in name:
            assert 0 < size <= 64, (name, size)
        else:
            assert size == 0, (name, size)
    # the plan reports the bound for that kernel and nothing for the others
    p = K.knn_plan(1_000_000, 1_000_000, 3, 16, 10 ** 9)
    assert p.path == K.KNN_PATH_LOWD_BF16 and p.private_bytes == 64 * 64 * 16 * 256
    assert p.workspace_bytes + p.private_bytes <= 10 ** 9
    assert K.knn_plan(2000, 100_000, 6, 16, 10 ** 9).private_bytes == 64 * 64 * 16 * 256  # path 4, d > 4
    assert K.knn_plan(2000, 100_000, 6, 16, 10 ** 7).private_bytes == 0  # no room: vector-ALU path
    assert K.knn_plan(100_000, 10_000_000, 128, 100, 8 * 10 ** 9).private_bytes == 0
    assert K.knn_plan(10_000, 1_000_000, 784, 10, 2 * 10 ** 9).private_bytes == 0
    # a limit with room for the packed points but not for the private segment beside them
    tight = K.knn_plan(1000, 200_000, 3, 16, 1 << 40)
    lim = tight.norms_bytes + 2 * 256 * 16 * 4 + 1000
    q = K.knn_plan(1000, 200_000, 3, 16, lim)
    assert q.path != K.KNN_PATH_LOWD_BF16 or q.workspace_bytes + q.private_bytes <= lim
