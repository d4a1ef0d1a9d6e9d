"""Compile the CPU oracle (gcc).  Run as ``python -m oracle.build``."""
from oracle import build

if __name__ == "__main__":
    print(build(force=True))
