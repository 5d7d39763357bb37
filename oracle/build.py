"""Compile the oracle's C source: ``python -m oracle.build``."""
from oracle import build

if __name__ == "__main__":
    print(build(force=True))
