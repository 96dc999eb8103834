"""CPU oracle (test infrastructure): see ckks.py / ckks_oracle.c."""
from .ckks import Oracle, build, gaussian_cdt  # noqa: F401
