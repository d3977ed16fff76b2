"""MI355X-native SpeCa sampling step: HIP kernels behind a C ABI (libspeca.so) and a thin
ctypes binding.  Importing the package does not load the library; the first call does, and
it fails loudly if the library has not been built."""
from . import binding  # noqa: F401
from .binding import (Context, Scheduler, SpecaError, load_library, make_cfg, cache_only_desc,  # noqa: F401
                      dit_desc, mmdit_desc, to_device)
