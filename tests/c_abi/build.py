"""Builds tests/c_abi/co2_selftest: a torch-free program that drives libco2.so through
the C ABI and checks it against the oracle source linked in (test infrastructure)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
EXE = os.path.join(HERE, "co2_selftest")


def build_selftest() -> str:
    pkg = os.path.join(ROOT, "paper_2401_16265_amd")
    oracle_obj = os.path.join(HERE, "oracle_for_selftest.o")
    subprocess.run(["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fno-fast-math", "-c",
                    os.path.join(ROOT, "oracle", "co2_oracle.cpp"), "-o", oracle_obj], check=True)
    # host-only program: g++ against the HIP runtime headers and library
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    subprocess.run(["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-D__HIP_PLATFORM_AMD__",
                    "-I", os.path.join(rocm, "include"), "-I", os.path.join(ROOT, "include"),
                    os.path.join(HERE, "selftest.cpp"), oracle_obj,
                    "-L", pkg, "-lco2", "-L", os.path.join(rocm, "lib"), "-lamdhip64",
                    "-Wl,-rpath," + pkg, "-Wl,-rpath," + os.path.join(rocm, "lib"), "-o", EXE],
                   check=True)
    return EXE


if __name__ == "__main__":
    print(build_selftest())
