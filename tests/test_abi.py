"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

from paper_2602_07223_amd import binding as vb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def good_desc(**over):
    kw = dict(batch=1, num_q_heads=32, num_kv_heads=8, num_queries=5, max_blocks=2048, max_sel_blocks=130,
              max_seq_len=32768, num_pages=2048, softmax_scale=128 ** -0.5)
    kw.update(over)
    fields = {k: kw.pop(k) for k in ("reserved",) if k in kw}       # descriptor fields make_desc has no argument for
    d = vb.make_desc(**kw)
    for k, v in fields.items():
        setattr(d, k, v)
    return d


def test_library_exports_every_declared_symbol():
    lib = vb.load_library()
    with open(os.path.join(ROOT, "include", "vegas.h")) as f:
        header = f.read()
    declared = set(re.findall(r"\b(vegas_[a-z_]+)\s*\(", header))
    assert declared == set(vb.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_desc_layout_matches_header():
    with open(os.path.join(ROOT, "include", "vegas.h")) as f:
        header = f.read()
    body = header[header.index("typedef struct vegas_desc {"):header.index("} vegas_desc;")]
    fields = re.findall(r"^\s*(?:int32_t|int64_t|float|void\*)\s+(\w+);", body, flags=re.M)
    assert fields == [f[0] for f in vb.VegasDesc._fields_]
    assert ctypes.sizeof(vb.VegasDesc) == 16 * 4 + 4 * 8           # 16 x 4-byte fields, 4 x 8-byte fields


def test_header_compiles_as_c_and_a_c_program_links_against_the_library(tmp_path):
    """include/vegas.h is a C header: a C11 compiler accepts it on its own, and a plain C program that includes it
    can call the pure-host entry points of the built library (struct layout and prototypes as the C side sees them)."""
    import shutil
    import subprocess
    cc = shutil.which("cc") or shutil.which("gcc")
    assert cc, "no C compiler"
    inc = os.path.join(ROOT, "include")
    r = subprocess.run([cc, "-std=c11", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", "-x", "c",
                        os.path.join(inc, "vegas.h")], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    src = tmp_path / "use_vegas.c"
    src.write_text(r'''
#include <stdio.h>
#include <string.h>
#include "vegas.h"
int main(void) {
  vegas_desc d;
  memset(&d, 0, sizeof d);
  d.batch = 1; d.num_q_heads = 32; d.num_kv_heads = 8; d.head_dim = 128; d.page_size = 16; d.num_queries = 5;
  d.max_blocks = 2048; d.max_sel_blocks = 130; d.max_seq_len = 32768; d.collect_rows = VEGAS_COLLECT_ALL_ROWS;
  d.softmax_scale = 0.08838834764831845f; d.score_metric = VEGAS_METRIC_PAGE_WEIGHTS;
  d.num_pages = 2048; d.kv_head_stride = 128; d.kv_token_stride = 1024; d.kv_page_stride = 16384;
  printf("%zu %zu\n", sizeof d, vegas_workspace_bytes(&d));
  d.head_dim = 96;
  printf("%zu\n", vegas_workspace_bytes(&d));
  printf("%s|%s\n", vegas_strerror(VEGAS_OK), vegas_strerror(VEGAS_ERR_WORKSPACE));
  /* argument validation comes before any launch: a NULL query is refused without touching a device */
  d.head_dim = 128;
  printf("%d\n", vegas_verify_attention(&d, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL));
  return 0;
}
''')
    exe = tmp_path / "use_vegas"
    libdir = os.path.dirname(vb.LIB_PATH)
    r = subprocess.run([cc, "-std=c11", "-Wall", "-Werror", "-I", inc, str(src), "-o", str(exe), "-L", libdir, "-lvegas",
                        "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stderr
    lines = r.stdout.split("\n")
    size, ws = lines[0].split()
    assert int(size) == ctypes.sizeof(vb.VegasDesc)
    assert int(ws) == vb.vegas_workspace_bytes(good_desc())
    assert lines[1] == "0"
    assert lines[2] == "ok|workspace missing or too small"
    assert int(lines[3]) == vb.VEGAS_ERR_NULL


def test_workspace_bytes_is_a_pure_host_function():
    n = vb.vegas_workspace_bytes(good_desc())
    assert n > 0 and n % 256 == 0
    assert vb.vegas_workspace_bytes(good_desc(max_seq_len=65536, max_blocks=4096)) > n
    assert 0 < vb.vegas_workspace_bytes(good_desc(head_dim=64)) < n     # partial rows are half as long
    assert vb.vegas_workspace_bytes(good_desc(head_dim=96)) == 0
    assert vb.vegas_workspace_bytes(good_desc(num_q_heads=30)) == 0


def test_strerror_is_defined_for_every_status():
    for s in range(0, -7, -1):
        assert vb.strerror(s) and vb.strerror(s) != "unknown status"
    assert vb.strerror(-99) == "unknown status"


A = 4096  # a 16-byte aligned fake device address: never dereferenced because validation fails first


@pytest.mark.parametrize("over,status", [
    (dict(batch=0), vb.VEGAS_ERR_SHAPE),
    (dict(num_q_heads=30), vb.VEGAS_ERR_SHAPE),
    (dict(head_dim=96), vb.VEGAS_ERR_UNSUPPORTED),
    (dict(page_size=32), vb.VEGAS_ERR_UNSUPPORTED),
    (dict(max_seq_len=32769), vb.VEGAS_ERR_SHAPE),
    (dict(num_queries=0), vb.VEGAS_ERR_SHAPE),
    (dict(num_queries=33), vb.VEGAS_ERR_UNSUPPORTED),          # 132 rows per KV head
    (dict(collect_rows=3), vb.VEGAS_ERR_SHAPE),
    (dict(kv_chunk_tokens=100), vb.VEGAS_ERR_SHAPE),
    (dict(kv_token_stride=1028), vb.VEGAS_ERR_ALIGN),
    (dict(softmax_scale=0.0), vb.VEGAS_ERR_SHAPE),
    (dict(batch=65536), vb.VEGAS_ERR_UNSUPPORTED),             # sequences are a grid dimension
    (dict(reserved=1), vb.VEGAS_ERR_SHAPE),
    (dict(max_seq_len=(1 << 30) + 16, max_blocks=(1 << 26) + 1), vb.VEGAS_ERR_UNSUPPORTED),
])
def test_verify_rejects_bad_descriptors(over, status):
    with pytest.raises(vb.VegasError) as e:
        vb.vegas_verify_attention(good_desc(**over), A, A, A, A, A, A, A, A, workspace_bytes=1 << 30)
    assert e.value.status == status


def test_verify_rejects_null_misaligned_and_small_workspace():
    d = good_desc()
    with pytest.raises(vb.VegasError) as e:
        vb.vegas_verify_attention(d, None, A, A, A, A, A, A, A, workspace_bytes=1 << 30)
    assert e.value.status == vb.VEGAS_ERR_NULL
    with pytest.raises(vb.VegasError) as e:
        vb.vegas_verify_attention(d, A, A, A, A, A, A, None, A, workspace_bytes=1 << 30)
    assert e.value.status == vb.VEGAS_ERR_NULL                  # scores required when collecting
    with pytest.raises(vb.VegasError) as e:
        vb.vegas_verify_attention(d, A + 2, A, A, A, A, A, A, A, workspace_bytes=1 << 30)
    assert e.value.status == vb.VEGAS_ERR_ALIGN
    with pytest.raises(vb.VegasError) as e:
        vb.vegas_verify_attention(d, A, A, A, A, A, A, A, A, workspace_bytes=1024)
    assert e.value.status == vb.VEGAS_ERR_WORKSPACE
    with pytest.raises(vb.VegasError) as e:
        vb.vegas_verify_attention(d, A, A, A, A, A, A, A, A + 16, workspace_bytes=1 << 30)
    assert e.value.status == vb.VEGAS_ERR_ALIGN


def test_select_and_draft_reject_bad_arguments():
    d = good_desc()
    with pytest.raises(vb.VegasError) as e:
        vb.vegas_select_blocks(d, A, A, A, 0, A, A)
    assert e.value.status == vb.VEGAS_ERR_SHAPE                 # budget must be positive
    with pytest.raises(vb.VegasError) as e:
        vb.vegas_select_blocks(d, A, A, A, 4096, A, A)
    assert e.value.status == vb.VEGAS_ERR_SHAPE                 # 256 pages do not fit max_sel_blocks=130
    with pytest.raises(vb.VegasError) as e:
        vb.vegas_select_blocks(d, None, A, A, 2048, A, A)
    assert e.value.status == vb.VEGAS_ERR_NULL
    with pytest.raises(vb.VegasError) as e:
        vb.vegas_draft_attention(d, A, A, A, A, A, A, A, workspace_bytes=1 << 30)
    assert e.value.status == vb.VEGAS_ERR_SHAPE                 # max_seq_len exceeds max_sel_blocks pages
    dd = good_desc(max_seq_len=130 * 16)
    with pytest.raises(vb.VegasError) as e:
        vb.vegas_draft_attention(dd, A, A, A, A, None, A, A, workspace_bytes=1 << 30)
    assert e.value.status == vb.VEGAS_ERR_NULL
    with pytest.raises(vb.VegasError) as e:
        vb.vegas_draft_attention(dd, A, A, A, A, A, A, None, workspace_bytes=0)
    assert e.value.status == vb.VEGAS_ERR_WORKSPACE


def test_static_scratch_refuses_what_does_not_fit():
    """A descriptor whose chunk partials exceed the built-in array is refused on the host, before any launch."""
    desc = vb.make_desc(batch=4096, num_q_heads=64, num_kv_heads=8, num_queries=1, max_blocks=64, max_sel_blocks=64,
                        max_seq_len=1024, num_pages=64, softmax_scale=0.1)
    assert vb.vegas_workspace_bytes(desc) > vb.vegas_static_scratch_bytes()
    with pytest.raises(vb.VegasError) as e:
        vb.vegas_draft_attention_static(desc, A, A, A, A, A, A)
    assert e.value.status == vb.VEGAS_ERR_WORKSPACE


def test_product_path_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2602_07223_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                with open(os.path.join(dirpath, fn)) as f:
                    text = f.read()
                assert not re.search(r"^\s*(from|import)\s+\S*oracle", text, flags=re.M), fn
                assert "vegas_oracle" not in text, fn
    for fn in os.listdir(os.path.join(ROOT, "oracle")):
        if fn.endswith(".py"):
            with open(os.path.join(ROOT, "oracle", fn)) as f:
                assert not re.search(r"^\s*(from|import)\s+paper_2602_07223_amd", f.read(), flags=re.M), fn


def test_binding_refuses_tensors_smaller_than_the_descriptor():
    """The C ABI sees bare pointers; the binding compares tensor extents with what the descriptor lets the
    kernels address and raises before anything reaches the library (CPU tensors here: nothing is launched)."""
    import torch
    d = good_desc(batch=2, max_blocks=8, max_sel_blocks=4, max_seq_len=100, num_pages=10)
    assert vb.cache_extent_bytes(d) == 10 * 16 * 8 * 128 * 2
    q = torch.zeros((2, 5, 32, 128), dtype=torch.bfloat16)
    cache = torch.zeros((10, 16, 8, 128), dtype=torch.bfloat16)
    half_width = torch.zeros((10, 16, 8, 64), dtype=torch.bfloat16)        # a head_dim-64 cache under a 128 descriptor
    table = torch.zeros((2, 8), dtype=torch.int32)
    lens = torch.zeros((2,), dtype=torch.int32)
    scores = torch.zeros((2, 8), dtype=torch.float32)
    ws = torch.zeros(vb.vegas_workspace_bytes(d), dtype=torch.uint8)
    with pytest.raises(ValueError, match="k_cache"):
        vb.vegas_verify_attention(d, q, half_width, cache, table, lens, torch.zeros_like(q), scores, ws)
    with pytest.raises(ValueError, match="v_cache"):
        vb.vegas_verify_attention(d, q, cache, cache[:9].clone(), table, lens, torch.zeros_like(q), scores, ws)
    with pytest.raises(ValueError, match="block_scores"):
        vb.vegas_verify_attention(d, q, cache, cache, table, lens, torch.zeros_like(q), scores[:1].clone(), ws)
    with pytest.raises(ValueError, match="out"):
        vb.vegas_verify_attention(d, q, cache, cache, table, lens, torch.zeros_like(q[:, :4]), scores, ws)
    sel = torch.zeros((2, 4), dtype=torch.int32)
    with pytest.raises(ValueError, match="sel_table"):
        vb.vegas_select_blocks(d, scores, table, lens, 32, sel[:, :3].contiguous(), lens.clone())
    with pytest.raises(ValueError, match="token_scores"):
        vb.vegas_select_tokens(d, scores, table, lens, 32, sel, lens.clone(), ws)
    qd = torch.zeros((2, 32, 128), dtype=torch.bfloat16)
    with pytest.raises(ValueError, match="k_cache"):
        vb.vegas_draft_attention(d, qd, half_width, cache, sel, lens, torch.zeros_like(qd), ws)
    # a strided view into a larger allocation is measured to the end of its storage
    big = torch.zeros((10, 16, 9, 192), dtype=torch.bfloat16)
    view = big[:, :, :8, :128]
    dv = good_desc(batch=2, max_blocks=8, max_sel_blocks=4, max_seq_len=100, num_pages=10,
                   kv_page_stride=view.stride(0), kv_token_stride=view.stride(1), kv_head_stride=view.stride(2))
    assert vb._avail_bytes(view) >= vb.cache_extent_bytes(dv)
    assert vb._avail_bytes(view[1:]) < vb.cache_extent_bytes(dv)


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU; bench.py says so and exits before touching a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and not r.stdout.strip()
