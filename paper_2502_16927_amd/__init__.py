"""MI355X-native BigMac MoE layer: a C-ABI HIP library (libbigmac.so) and a thin ctypes binding."""
from . import synth  # noqa: F401
