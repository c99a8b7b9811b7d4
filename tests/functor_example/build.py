"""Build the user-side examples of the functor hooks (sine_flux.hip -> libsine_flux.so,
star_bodies.hip -> libstar_bodies.so; gfx950)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
LIB = os.path.join(HERE, "libsine_flux.so")
LIB_STAR = os.path.join(HERE, "libstar_bodies.so")


def _compile(src: str, lib: str) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = lib + ".tmp%d" % os.getpid()
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall",
                           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                           "-I", os.path.join(ROOT, "include"),
                           os.path.join(HERE, src), "-o", tmp])
    os.replace(tmp, lib)
    return lib


def build() -> str:
    _compile("star_bodies.hip", LIB_STAR)
    return _compile("sine_flux.hip", LIB)


if __name__ == "__main__":
    print(build())
