"""A checkout that holds only the tracked files must build: __graft_entry__.build() compiles
libcard.so with nothing prebuilt beside it, and the result loads and exports the C ABI."""
import ctypes
import os
import re
import shutil
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _tracked_files():
    out = subprocess.run(["git", "ls-files", "-co", "--exclude-standard"], cwd=ROOT, capture_output=True, text=True)
    if out.returncode != 0 or not out.stdout.strip():
        return None
    return [f for f in out.stdout.splitlines() if os.path.isfile(os.path.join(ROOT, f))]


def test_build_from_tracked_files_only(tmp_path):
    files = _tracked_files()
    if files is None:  # not a git checkout (e.g. an exported tree): take the source folders as they are
        files = []
        for top in ("include", "paper_2508_04462_amd", "oracle", "card_inputs"):
            for d, _, names in os.walk(os.path.join(ROOT, top)):
                files += [os.path.relpath(os.path.join(d, n), ROOT) for n in names]
        files.append("__graft_entry__.py")
    # no built artefact travels, whatever the ignore rules say
    files = [f for f in files if not f.endswith((".so", ".o", ".pyc")) and not f.startswith(("tests/", "profiles/", "_work/"))]
    assert "__graft_entry__.py" in files and "paper_2508_04462_amd/csrc/card_api.hip" in files
    for f in files:
        dst = tmp_path / f
        dst.parent.mkdir(parents=True, exist_ok=True)
        shutil.copyfile(os.path.join(ROOT, f), dst)
    lib = tmp_path / "paper_2508_04462_amd" / "libcard.so"
    assert not lib.exists()
    env = {k: v for k, v in os.environ.items() if k != "PYTHONPATH"}
    p = subprocess.run([sys.executable, "-c", "import __graft_entry__ as g; g.build(); "
                        "import paper_2508_04462_amd as c; print(c.card_strerror(-3))"],
                       cwd=tmp_path, env=env, capture_output=True, text=True, timeout=900)
    assert p.returncode == 0, p.stderr[-2000:]
    assert "KV cache capacity exceeded" in p.stdout
    assert lib.exists()
    cdll = ctypes.CDLL(str(lib))
    header = open(os.path.join(ROOT, "include", "card.h")).read()
    for name in sorted(set(re.findall(r"\b(card_[a-z_]+)\s*\(", header))):
        assert hasattr(cdll, name), name


def test_missing_library_fails_loudly_at_first_use(tmp_path):
    """No fallback: with no libcard.so beside the binding the first entry point raises."""
    pkg = tmp_path / "paper_2508_04462_amd"
    pkg.mkdir()
    for f in os.listdir(os.path.join(ROOT, "paper_2508_04462_amd")):
        if f.endswith(".py"):
            shutil.copyfile(os.path.join(ROOT, "paper_2508_04462_amd", f), pkg / f)
    shutil.copytree(os.path.join(ROOT, "card_inputs"), tmp_path / "card_inputs")
    env = {k: v for k, v in os.environ.items() if k != "PYTHONPATH"}
    code = ("import paper_2508_04462_amd as c\n"
            "try:\n    c.card_strerror(0)\nexcept ImportError as e:\n    print('LOUD', e)\n")
    p = subprocess.run([sys.executable, "-c", code], cwd=tmp_path, env=env, capture_output=True, text=True, timeout=300)
    assert p.returncode == 0, p.stderr[-2000:]
    assert "LOUD" in p.stdout and "libcard.so is missing" in p.stdout
