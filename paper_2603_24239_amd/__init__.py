"""MI355X-native bytecode virtual machine for fused dynamic-shape tensor programs (libdvm)."""
from . import binding  # noqa: F401
