"""Child process of test_oracle_mutants: load a (deliberately broken) oracle build,
run every pin, exit 3 as soon as one fails, 0 if none does.  Run as
``python -m tests.mutant_runner <path/to/mutant.so>`` from the repository root.
A planted mistake may also corrupt host memory and crash this process; the parent
counts that as noticed, which is why the pins run out of process."""
import ctypes
import sys


def main(so_path: str) -> int:
    import oracle
    from tests import test_oracle_pins as pins

    real = oracle.lib()
    mutant = ctypes.CDLL(so_path)
    for fn in ("orc_f32_to_bf16", "orc_bf16_to_f32"):
        getattr(mutant, fn).restype = getattr(real, fn).restype
        getattr(mutant, fn).argtypes = getattr(real, fn).argtypes
    oracle._lib = mutant
    for check in pins.ALL_CHECKS:
        try:
            check()
        except AssertionError:
            print(f"caught by {check.__name__}")
            return 3
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1]))
