"""Builds nfad_c_check (the plain-C exerciser of the C ABI) next to its source, with gcc.

It links libnfad.so (the product), libnfad_oracle.so (the yardstick) and the HIP runtime's C
API; run-time library paths are relative to the binary, so the tree can be moved."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
BINARY = os.path.join(HERE, "nfad_c_check")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build() -> str:
    libnfad = os.path.join(ROOT, "paper_2209_10778_amd", "libnfad.so")
    liboracle = os.path.join(ROOT, "oracle", "libnfad_oracle.so")
    for lib in (libnfad, liboracle):
        if not os.path.exists(lib):
            raise FileNotFoundError(f"{lib} is missing: build the library and the oracle first")
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-Werror", f"-I{os.path.join(ROOT, 'include')}", f"-I{ROCM}/include",
           os.path.join(HERE, "nfad_c_check.c"), "-o", BINARY, libnfad, liboracle,
           f"-L{ROCM}/lib", "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN/../../paper_2209_10778_amd", "-Wl,-rpath,$ORIGIN/../../oracle",
           f"-Wl,-rpath,{ROCM}/lib"]
    subprocess.run(cmd, check=True)
    return BINARY


if __name__ == "__main__":
    print(build())
