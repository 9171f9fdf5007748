"""`python -m oracle.build` compiles oracle/dream_oracle.c into oracle/liboracle.so with gcc."""
from . import build

if __name__ == "__main__":
    print(build(force=True))
