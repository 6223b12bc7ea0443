"""Compile the CPU oracle into oracle/libssnet_oracle.so (gcc, OpenMP).

Test infrastructure only: nothing in the GPU library links against this.

A second target, oracle/libssnet_oracle_san.so, is the same source under
AddressSanitizer and UndefinedBehaviorSanitizer (-O1 -g, a finding aborts).  With
SSNET_ORACLE_SANITIZED=1 in the environment the oracle module loads that one; the
interpreter then has to start with the sanitizer runtime preloaded, see
sanitizer_env().  tests/test_oracle_sanitized.py runs the oracle's pins that way.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "ssnet_oracle.c")
LIB = os.path.join(HERE, "libssnet_oracle.so")
LIB_SAN = os.path.join(HERE, "libssnet_oracle_san.so")


def build(force: bool = False) -> str:
    if (not force and os.path.exists(LIB)
            and os.path.getmtime(LIB) >= os.path.getmtime(SRC)):
        return LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", LIB + ".tmp", SRC, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(LIB + ".tmp", LIB)
    return LIB


def sanitizer_runtime() -> str:
    """path of gcc's libasan.so, '' if this toolchain has none"""
    r = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True)
    path = r.stdout.strip()
    return path if r.returncode == 0 and os.path.isabs(path) and os.path.exists(path) else ""


def build_sanitized(force: bool = False) -> str:
    if (not force and os.path.exists(LIB_SAN)
            and os.path.getmtime(LIB_SAN) >= os.path.getmtime(SRC)):
        return LIB_SAN
    cmd = ["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fopenmp", "-shared", "-fPIC", "-o", LIB_SAN + ".tmp", SRC, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(LIB_SAN + ".tmp", LIB_SAN)
    return LIB_SAN


def sanitizer_env(env=None) -> dict:
    """environment for a child interpreter that loads the sanitized oracle: the sanitizer runtime preloaded behind
    whatever is preloaded already, leak checking off (the interpreter itself never frees everything)"""
    env = dict(os.environ if env is None else env)
    pre = [x for x in env.get("LD_PRELOAD", "").replace(":", " ").split() if x]
    env["LD_PRELOAD"] = " ".join(pre + [sanitizer_runtime()])
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["SSNET_ORACLE_SANITIZED"] = "1"
    return env


if __name__ == "__main__":
    print(build(force=True))
    if sanitizer_runtime():
        print(build_sanitized(force=True))
