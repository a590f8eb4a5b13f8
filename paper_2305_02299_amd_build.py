"""Build entry used before the package can be imported (the package import needs libsrigl.so)."""
import importlib.util
import os

ROOT = os.path.dirname(os.path.abspath(__file__))


def build_all(verbose: bool = False) -> None:
    spec = importlib.util.spec_from_file_location("_srigl_build", os.path.join(ROOT, "paper_2305_02299_amd", "build.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod.build(verbose=verbose)
    import oracle
    oracle.build(force=True)
