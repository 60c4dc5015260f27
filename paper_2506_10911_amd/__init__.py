"""NoLoCo outer optimizer step for AMD MI355X (arxiv 2506.10911, Eq. 1-3).

The work is done by hand-written HIP kernels behind the C ABI of include/noloco.h; this
package is the thin Python binding to it (argument marshalling only). The binding, and with
it libnoloco.so, is loaded on first use of any name below, so that
`python -m paper_2506_10911_amd.build` can run before the library exists. There is no
fallback: if the library is missing, that first use raises.
"""
_NAMES = ("BF16", "F32", "LaunchPlan", "NolocoError", "copy_probe", "fill_probe", "read_probe",
          "library_path", "merge_segments", "outer_step", "plan_groups", "plan_routes", "replica_spread", "replica_spread_noalloc", "sim_tree_vs_pair", "sim_barrier_penalty", "strerror",
          "binding")


def __getattr__(name):
    if name in _NAMES:
        import importlib
        binding = importlib.import_module(".binding", __name__)
        return binding if name == "binding" else getattr(binding, name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")


def __dir__():
    return sorted(list(globals()) + list(_NAMES))
