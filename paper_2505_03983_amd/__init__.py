"""MI355X-native Autospeculative Decoding (ASD) for DDPM sampling.

The product is the HIP library `libasd.so` (sources under `csrc/`, C boundary
in `include/asd.h`); `binding` is its ctypes wrapper and `runtime` sets a
workload up on the device."""
