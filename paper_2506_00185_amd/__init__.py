"""MI355X-native batched beam search for RNN-T / TDT Transducers (ALSD++ / AES++).

The work is done by ``librnnt_beam.so`` (HIP kernels behind a C ABI, declared in
``include/rnnt_beam.h``).  This package is the thin binding: it marshals
arguments and uses PyTorch only to hold device memory and streams.  There is no
CPU fallback: without the built library every call raises.
"""
from .binding import (ALSD, AES, BeamDecoder, NGramLM, RnntBeamError, library_path, load_library)  # noqa: F401
