"""MI355X-native selective-SSM layer core of a Mamba drafter (gfx950 HIP kernels behind a C ABI).

``paper_2506_01206_amd.binding`` holds the ctypes binding of the C-ABI library
(mamba_conv1d_fwd, mamba_scan_fwd, mamba_state_step, mamba_state_fork);
``paper_2506_01206_amd.synth`` the seeded input generators.  The binding is
imported on first attribute access so that the generators stay usable where
the library has not been built; using any kernel without it raises.
"""
from . import synth  # noqa: F401

_BINDING_NAMES = ("mamba_conv1d_fwd", "mamba_scan_fwd", "mamba_scan_workspace_bytes",
                  "mamba_state_step", "mamba_state_fork", "mamba_status_string", "mamba_tree_plan",
                  "mamba_tree_parents", "mamba_linear_fwd", "mamba_rmsnorm_fwd", "binding")


def __getattr__(name):
    if name in _BINDING_NAMES:
        import importlib
        b = importlib.import_module(__name__ + ".binding")
        return b if name == "binding" else getattr(b, name)
    raise AttributeError(name)
