"""Compile tests/c_abi_check.c: a plain-C user of the GPU library, with the C oracle linked in
as its checker.  Both shared libraries must exist already."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def build_c_check(verbose=False) -> str:
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    src, out = os.path.join(HERE, "c_abi_check.c"), os.path.join(HERE, "c_abi_check")
    inc, pkg, orc = os.path.join(ROOT, "include"), os.path.join(ROOT, "paper_2504_17307_amd"), os.path.join(ROOT, "oracle")
    cmd = ["gcc", "-O1", "-std=c11", "-Wall", "-D__HIP_PLATFORM_AMD__", f"-I{rocm}/include", f"-I{inc}", f"-I{orc}",
           src, f"-L{pkg}", "-luccl_chunk", f"-L{orc}", "-lchunk_oracle", f"-L{rocm}/lib", "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../paper_2504_17307_amd", "-Wl,-rpath,$ORIGIN/../oracle", f"-Wl,-rpath,{rocm}/lib",
           "-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return out


if __name__ == "__main__":
    print(build_c_check(verbose=True))
