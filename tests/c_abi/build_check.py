"""Builds tests/c_abi/c_abi_check (plain C against libbiq.so and the C oracle).  Test infrastructure."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
SRC = os.path.join(HERE, "c_abi_check.c")
EXE = os.path.join(HERE, "c_abi_check")


def build() -> str:
    """Needs paper_2005_09904_amd/libbiq.so and oracle/libbiq_oracle.so to exist (linked by path,
    found again at run time through $ORIGIN-relative rpaths)."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    pkg = os.path.join(ROOT, "paper_2005_09904_amd")
    orc = os.path.join(ROOT, "oracle")
    tmp = EXE + ".tmp.%d" % os.getpid()
    # plain C compiler; the HIP headers want to be told the platform when it is not hipcc
    cmd = ["gcc", "-O1", "-std=c99", "-D__HIP_PLATFORM_AMD__", "-I" + os.path.join(rocm, "include"),
           "-I" + os.path.join(ROOT, "include"), SRC, "-o", tmp,
           "-L" + os.path.join(rocm, "lib"), "-lamdhip64", "-Wl,-rpath," + os.path.join(rocm, "lib"),
           "-L" + pkg, "-l:libbiq.so", "-L" + orc, "-l:libbiq_oracle.so", "-lm",
           "-Wl,-rpath,$ORIGIN/../../paper_2005_09904_amd", "-Wl,-rpath,$ORIGIN/../../oracle"]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        if os.path.exists(tmp):
            os.remove(tmp)
        raise RuntimeError("building c_abi_check failed:\n" + proc.stdout)
    os.replace(tmp, EXE)
    return EXE


if __name__ == "__main__":
    print(build())
