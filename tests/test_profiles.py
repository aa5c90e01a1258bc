"""bench.py may quote counter traffic only from a profile summary made for exactly the workload,
feature width, plan options and library sources it is timing (paper_2603_08734_amd/profiles.py)."""
import json

from paper_2603_08734_amd import build, profiles


def _write(dirname, name, **over):
    data = {"workload": "w", "N": 128, "plan_options": {}, "library_sources": build.source_digest(),
            "bench_args": "--config 2",
            "kernels": {"rsh::rsh_irregular_kernel<16, rsh::OutFused, false>": {"fetched_bytes": 7, "written_bytes": 1},
                        "rsh::rsh_irregular_kernel<16, rsh::OutPlain, false>": {"fetched_bytes": 100, "written_bytes": 20},
                        "rsh::rsh_combine_kernel<rsh::OutPlain>": {"fetched_bytes": 5, "written_bytes": 5}}}
    data.update(over)
    (dirname / name).write_text("# summary\n\n" + profiles._MARK + "\n```json\n" + json.dumps(data) + "\n```\n")


def test_lookup_matches_workload_width_options_and_sources(tmp_path, monkeypatch):
    monkeypatch.setattr(profiles, "PROFILE_DIR", str(tmp_path))
    _write(tmp_path, "a.md")
    (tmp_path / "notes.md").write_text("no data block here\n")
    got = profiles.lookup("w", 128, {}, "rsh_irregular_kernel")
    assert got == (120, "a.md", "rsh::rsh_irregular_kernel<16, rsh::OutPlain, false>")
    assert profiles.lookup("w", 64, {}, "rsh_irregular_kernel") is None
    assert profiles.lookup("other", 128, {}, "rsh_irregular_kernel") is None
    assert profiles.lookup("w", 128, {"min_reuse": "1.0"}, "rsh_irregular_kernel") is None
    assert profiles.lookup("w", 128, {}, "rsh_tile_kernel") is None


def test_lookup_refuses_a_summary_of_other_sources(tmp_path, monkeypatch):
    monkeypatch.setattr(profiles, "PROFILE_DIR", str(tmp_path))
    _write(tmp_path, "a.md", library_sources="0" * 64)
    assert profiles.lookup("w", 128, {}, "rsh_irregular_kernel") is None


def test_lookup_prefers_the_plain_command(tmp_path, monkeypatch):
    monkeypatch.setattr(profiles, "PROFILE_DIR", str(tmp_path))
    _write(tmp_path, "a_epilogue.md", bench_args="--config 2 --epilogue")
    _write(tmp_path, "b.md")
    assert profiles.lookup("w", 128, {}, "rsh_irregular_kernel")[1] == "b.md"


def test_committed_summaries_parse():
    names = [name for name, data in profiles._blocks() if {"workload", "N", "plan_options", "kernels"} <= set(data)]
    assert names, "profiles/ holds no summary in the format bench.py reads"
