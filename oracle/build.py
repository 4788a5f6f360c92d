"""Compile the C oracle: `python -m oracle.build`."""
from .forward import build

if __name__ == "__main__":
    print(build(force=True))
