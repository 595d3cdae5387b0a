"""Host-only checks of the C-ABI library: it loads without a GPU, exports every symbol
include/mw.h declares, its records have the documented sizes and offsets, and the
host-side validation answers without touching a device."""
import ctypes as C
import os
import re
import subprocess
import tempfile

import numpy as np
import pytest

from paper_2605_22428_amd import binding as B
from paper_2605_22428_amd import build as hip_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "mw.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        hip_build.build()
    return B.load()


def test_exports_every_declared_symbol(lib):
    text = open(HEADER).read()
    declared = re.findall(r"MW_API\s+[\w\s\*]+?\b(mw_\w+)\s*\(", text)
    assert sorted(set(declared)) == sorted(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_record_layouts_match_the_header():
    src = r'''
#include <stdio.h>
#include <stddef.h>
#include "mw.h"
int main(void) {
  printf("%zu %zu %zu %zu %zu\n", sizeof(mw_group_desc), sizeof(mw_send_stats), sizeof(mw_recv_stats),
         sizeof(mw_recv_peer), sizeof(mw_config));
  printf("%zu %zu %zu %zu\n", sizeof(mw_relay_child), sizeof(mw_relay_stats), offsetof(mw_relay_stats, rows_per_hop),
         offsetof(mw_relay_stats, error_flags));
  printf("%zu %zu %zu\n", offsetof(mw_group_desc, row_offset), offsetof(mw_group_desc, n_dest),
         offsetof(mw_send_stats, rows_per_dest));
  printf("%zu %zu %zu %zu\n", offsetof(mw_send_stats, error_flags), offsetof(mw_recv_peer, rows),
         offsetof(mw_recv_peer, row_topk), offsetof(mw_config, expert_to_rank));
  return 0; }
'''
    with tempfile.TemporaryDirectory() as d:
        c = os.path.join(d, "t.c")
        open(c, "w").write(src)
        exe = os.path.join(d, "t")
        subprocess.check_call(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), c, "-o", exe])
        out = subprocess.check_output([exe]).decode().split()
    vals = [int(v) for v in out]
    assert vals[:5] == [48, 1056, 24, 40, C.sizeof(B.MwConfig)]
    assert vals[5:9] == [32, 544, B.RELAY_STATS_DTYPE.fields["rows_per_hop"][1],
                         B.RELAY_STATS_DTYPE.fields["error_flags"][1]]
    vals = vals[:5] + vals[9:]
    assert vals[5:8] == [B.DESC_DTYPE.fields["row_offset"][1], B.DESC_DTYPE.fields["n_dest"][1],
                         B.SEND_STATS_DTYPE.fields["rows_per_dest"][1]]
    assert vals[8:] == [B.SEND_STATS_DTYPE.fields["error_flags"][1], B.RECV_PEER_DTYPE.fields["rows"][1],
                        B.RECV_PEER_DTYPE.fields["row_topk"][1], B.MwConfig.expert_to_rank.offset]


def test_batch_records_match_the_header():
    """mw_send_batch, mw_recv_batch, mw_next_batch, mw_relay_job: the binding's ctypes records have the size and
    the member offsets the C compiler gives the header's."""
    recs = [("mw_send_batch", B.MwSendBatch), ("mw_recv_batch", B.MwRecvBatch), ("mw_next_batch", B.MwNextBatch),
            ("mw_relay_job", B.MwRelayJob)]
    lines = []
    for cname, cls in recs:
        lines.append('printf("%%zu", sizeof(%s));' % cname)
        for f, _ in cls._fields_:
            lines.append('printf(" %%zu", offsetof(%s, %s));' % (cname, f))
        lines.append('printf("\\n");')
    src = "#include <stdio.h>\n#include <stddef.h>\n#include \"mw.h\"\nint main(void) {\n%s\nreturn 0; }\n" % "\n".join(lines)
    with tempfile.TemporaryDirectory() as d:
        c = os.path.join(d, "t.c")
        open(c, "w").write(src)
        exe = os.path.join(d, "t")
        subprocess.check_call(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), c, "-o", exe])
        out = subprocess.check_output([exe]).decode().splitlines()
    assert len(out) == len(recs)
    for line, (cname, cls) in zip(out, recs):
        vals = [int(v) for v in line.split()]
        assert vals[0] == C.sizeof(cls), cname
        assert vals[1:] == [getattr(cls, f).offset for f, _ in cls._fields_], cname
    assert (C.sizeof(B.MwSendBatch), C.sizeof(B.MwRecvBatch), C.sizeof(B.MwNextBatch), C.sizeof(B.MwRelayJob)) == (72, 48, 88, 40)


def _cfg(**kw):
    e2r = np.arange(16, dtype=np.int32) // 2
    base = dict(n_ranks=8, n_experts=16, top_k=2, my_rank=0, hidden=256, row_format=B.MW_ROW_BF16,
                row_bytes=0, max_tokens=128, max_hops=0, max_recv_rows=1024,
                expert_to_rank=e2r.ctypes.data)
    base.update(kw)
    return B.MwConfig(**base), e2r


def test_workspace_query_and_validation(lib):
    need = C.c_int64(0)
    cfg, keep = _cfg()
    assert lib.mw_workspace_bytes(C.byref(cfg), C.byref(need)) == B.MW_OK and need.value > 0
    assert need.value % 256 == 0
    for kw, want in [(dict(n_ranks=257), B.MW_ERR_UNSUPPORTED),          # bitmap is 256 bits wide
                     (dict(top_k=65), B.MW_ERR_UNSUPPORTED),
                     (dict(my_rank=8), B.MW_ERR_INVALID_ARG),
                     (dict(top_k=0), B.MW_ERR_INVALID_ARG),
                     (dict(hidden=7), B.MW_ERR_UNSUPPORTED),              # 14-byte rows
                     (dict(row_format=B.MW_ROW_FP8_E4M3_BLOCK128, hidden=256), B.MW_ERR_UNSUPPORTED),
                     (dict(row_format=B.MW_ROW_FP8_E4M3_BLOCK128, hidden=7168), B.MW_OK),
                     (dict(row_format=B.MW_ROW_BYTES, row_bytes=24), B.MW_ERR_UNSUPPORTED),
                     (dict(row_format=B.MW_ROW_BYTES, row_bytes=2 << 20), B.MW_OK),
                     (dict(row_bytes=100), B.MW_ERR_INVALID_ARG),         # contradicts the bf16 row size
                     (dict(max_tokens=1 << 20), B.MW_ERR_UNSUPPORTED),
                     (dict(max_hops=65), B.MW_ERR_UNSUPPORTED),
                     (dict(max_hops=-1), B.MW_ERR_INVALID_ARG),
                     (dict(max_hops=16), B.MW_OK),
                     (dict(expert_to_rank=0), B.MW_ERR_INVALID_ARG)]:
        cfg, keep = _cfg(**kw)
        assert lib.mw_workspace_bytes(C.byref(cfg), C.byref(need)) == want, kw
    bad = np.full(16, 9, dtype=np.int32)
    cfg, keep = _cfg(expert_to_rank=bad.ctypes.data)
    assert lib.mw_workspace_bytes(C.byref(cfg), C.byref(need)) == B.MW_ERR_INVALID_ARG
    assert lib.mw_workspace_bytes(None, C.byref(need)) == B.MW_ERR_INVALID_ARG
    # a context needs a workspace: rejected before any device call
    cfg, keep = _cfg()
    h = C.c_void_p(0)
    assert lib.mw_ctx_create(C.byref(cfg), None, C.c_int64(0), C.byref(h)) == B.MW_ERR_WORKSPACE


def test_status_strings(lib):
    assert B.status_string(0) == "ok"
    for s in (-1, -2, -3, -4, -5):
        assert B.status_string(s) not in ("ok", "unknown status")
    assert B.status_string(-99) == "unknown status"


def test_allgather_split_point_is_host_arithmetic(lib):
    """No device involved: the split point follows Section 3.1's two-path model; compared with
    the oracle's own formula and with the two cases the paper works out."""
    from oracle import ref
    s = 16 << 20
    assert B.mw_allgather_split_point(s, 1.0, 1.0, 1) == s // 2        # multicast: half and half
    assert B.mw_allgather_split_point(s, 1.0, 1.0, 3) == 3 * s // 4    # unicast multi-path to 3 peers
    for args in [(s, 56.0, 25.0, 1), (2 << 20, 3.0, 7.0, 2), (4096, 1.0, 1000.0, 1), (0, 1.0, 1.0, 1),
                 (48, 1.0, 1.0, 1)]:
        assert B.mw_allgather_split_point(*args) == ref.allgather_split_point(*args)
    for args, want in [((s + 8, 1.0, 1.0, 1), B.MW_ERR_UNSUPPORTED), ((s, 0.0, 1.0, 1), B.MW_ERR_INVALID_ARG),
                       ((s, 1.0, 1.0, 0), B.MW_ERR_INVALID_ARG), ((-16, 1.0, 1.0, 1), B.MW_ERR_INVALID_ARG)]:
        with pytest.raises(B.MwError) as e:
            B.mw_allgather_split_point(*args)
        assert e.value.status == want
