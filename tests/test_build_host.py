"""Host-side checks of the build script's incremental rule (no compiler is run)."""
import os

from paper_2212_05191_amd import build as B


def _touch(path, mtime):
    with open(path, "w") as f:
        f.write("x")
    os.utime(path, (mtime, mtime))


def test_incremental_build_recompiles_objects_older_than_a_header(tmp_path):
    # objects share struct layouts through the headers: one compiled before a header changed must not be linked
    srcs = ["a.hip", "b.hip", "c.hip", "d.hip"]
    objs = [str(tmp_path / s.replace(".hip", ".o")) for s in srcs]
    old_h, new_h = str(tmp_path / "old.hpp"), str(tmp_path / "new.hpp")
    _touch(old_h, 1000)
    _touch(new_h, 2000)
    _touch(objs[0], 1500)    # asked for anyway
    _touch(objs[1], 1500)    # older than new.hpp: stale
    _touch(objs[2], 2500)    # newer than every header: kept
    # objs[3] does not exist: compiled
    got = B.sources_to_compile(["a.hip"], srcs, objs, [old_h, new_h])
    assert got[0] == "a.hip" and sorted(got) == ["a.hip", "b.hip", "d.hip"]


def test_incremental_build_keeps_fresh_objects_and_passes_other_names_through(tmp_path):
    srcs = ["a.hip", "b.hip"]
    objs = [str(tmp_path / "a.o"), str(tmp_path / "b.o")]
    hdr = str(tmp_path / "h.hpp")
    _touch(hdr, 1000)
    _touch(objs[0], 2000)
    _touch(objs[1], 2000)
    assert B.sources_to_compile(["peaks_probe.hip"], srcs, objs, [hdr]) == ["peaks_probe.hip"]
    assert B.sources_to_compile([], srcs, objs, [hdr]) == []
    os.utime(hdr, (3000, 3000))
    assert sorted(B.sources_to_compile([], srcs, objs, [hdr])) == ["a.hip", "b.hip"]


def test_every_source_of_the_library_exists_and_every_hip_file_is_built():
    on_disk = {f for f in os.listdir(B.CSRC) if f.endswith(".hip")}
    assert set(B.SOURCES) | {"peaks_probe.hip"} == on_disk
    assert "-packed-fp32-ops" in B.FLAGS and "--offload-arch=gfx950" in B.FLAGS
