"""The C-ABI library loads without a GPU and exports every function the headers declare."""
import glob
import os
import re

import paper_2605_23945_amd as pat

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    for h in glob.glob(os.path.join(ROOT, "include", "*.h")):
        text = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)          # drop comments
        # a declaration: return type, name, '(' ... ');' at file scope
        for m in re.finditer(r"^[A-Za-z_][\w\s\*]*?\b(pat_\w+)\s*\(", text, flags=re.M):
            names.add(m.group(1))
    return names


def test_every_declared_function_is_exported_and_bound():
    lib = pat.load_library()
    declared = _declared()
    assert len(declared) >= 30, declared
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} is declared in include/ but not exported by the library"
    assert declared == set(pat.EXPORTS), (declared ^ set(pat.EXPORTS))


def test_host_only_calls_reject_bad_arguments_without_a_gpu():
    lib = pat.load_library()
    assert lib.pat_op_gemm_scratch_bytes(0, 64, 1) == -1
    assert lib.pat_op_packed_weight_bytes(16, 33) < 0          # k not a multiple of 32
    cfg = pat.pat_cfg()
    req = pat.pat_mem_req()
    assert lib.pat_decode_query(cfg, req) == pat.binding.PAT_EINVAL


def test_static_scratch_entry_point_refuses_oversized_partial_sums_without_a_gpu():
    """pat_op_gemm_static checks the size of the K-slice partial sums before any GPU call."""
    lib = pat.load_library()
    n, k, b = 22016, 4096, 256
    assert lib.pat_op_gemm_scratch_bytes(n, k, b) > (32 << 20)
    one = 0x1000                                                 # never dereferenced: the call fails first
    assert lib.pat_op_gemm_static(one, n, k, one, one, b, one, n, None, None, 0, None) == pat.binding.PAT_ENOMEM
    assert lib.pat_op_gemm_static(None, n, k, one, one, b, one, n, None, None, 0, None) == pat.binding.PAT_EINVAL
