
from . import build, measure

if __name__ == "__main__":
    build()
    for k, v in measure().items():
        print(f"{k:32s} {v}")
