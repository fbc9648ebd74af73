"""MI355X-native JoT token-finalization pass: a C-ABI HIP library plus this thin binding.

All computation happens in the HIP library (csrc/); there is no CPU or framework fallback.
Importing the package does not load the library; the first call does, and raises if the library
has not been built (see build.py)."""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
