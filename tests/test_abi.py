"""The C-ABI library loads and exports every symbol the headers under include/ declare (no GPU, no compute)."""
import glob
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    import paper_2410_13333_amd as mls
    headers = sorted(glob.glob(os.path.join(ROOT, "include", "*.h")))
    assert [os.path.basename(h) for h in headers] == ["mls.h", "mls_ends.h", "mls_optim.h", "mls_plan.h"]
    header = "".join(open(h).read() for h in headers)
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(mls_[a-z_]+)\s*\(", header))
    assert {"mls_stage_init", "mls_stage_forward", "mls_stage_backward", "mls_stage_free", "mls_plan_layers",
            "mls_plan_microbatches", "mls_plan_lower_level", "mls_embed_forward", "mls_embed_backward",
            "mls_head_forward", "mls_head_backward", "mls_optim_step", "mls_probe_read"} <= names
    lib = ctypes.CDLL(mls.lib_path())
    for n in sorted(names):
        assert hasattr(lib, n), n


def test_config_struct_matches_header_field_order():
    import paper_2410_13333_amd as mls
    header = open(os.path.join(ROOT, "include", "mls.h")).read()
    body = header[header.index("typedef struct {"):header.index("} mls_config;")]
    fields = re.findall(r"^\s*(?:int32_t|float)\s+(\w+);", body, flags=re.M)
    assert fields == [f[0] for f in mls.MlsConfig._fields_]
    assert ctypes.sizeof(mls.MlsConfig) == 52


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2410_13333_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.replace("no fallback", ""), f
