"""`python -m oracle.build` compiles oracle/dream_oracle.c into oracle/liboracle.so with gcc.
`python -m oracle.build --sanitize` builds the host sanitizer variants as well and runs the AddressSanitizer self-test
(see oracle.build_sanitized); `DREAM_ORACLE_UBSAN=1 python -m pytest tests -m "not gpu"` then runs the CPU suite on the
UBSan library."""
import sys

from . import build, build_sanitized

if __name__ == "__main__":
    print(build(force=True))
    if "--sanitize" in sys.argv[1:]:
        r = build_sanitized(run_selftest=True)
        print(r["selftest"], r["library"])
        print(r["selftest_output"].strip())
