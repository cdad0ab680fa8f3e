"""MI355X-native draft-tree verification (the target verification pass of
cascaded tree speculation).  All computation lives in libcats.so (HIP, gfx950);
this package only marshals arguments.  Importing it does not load the library;
the first call does, and fails loudly if the library has not been built."""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
