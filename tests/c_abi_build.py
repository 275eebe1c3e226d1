"""Compile tests/c_abi_client.c (a plain C consumer of include/vla.h) with gcc against the built libvla.so and
the HIP runtime.  Called from __graft_entry__.build(); the binary is looked up by tests/test_c_abi_gpu.py."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "c_abi_client.c")
OUT = os.path.join(HERE, "c_abi_client")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build(verbose: bool = False) -> str:
    libdir = os.path.join(HERE, "..", "paper_2605_11196_amd")
    cmd = ["gcc", "-std=c11", "-O1", "-Wall", "-Wextra", "-D__HIP_PLATFORM_AMD__", f"-I{ROCM}/include", SRC,
           "-o", OUT, f"-L{libdir}", "-lvla", f"-L{ROCM}/lib", "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../paper_2605_11196_amd", f"-Wl,-rpath,{ROCM}/lib"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    print(build(verbose=True))
