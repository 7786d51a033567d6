"""MI355X-native shuffle pipeline of compressed coded distributed computing.

`binding` mirrors the C entry points of libccdc.so (include/ccdc.h); `build`
compiles the library in-tree.  Importing the package does not load the
library; the first use does, and fails loudly if it has not been built.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    CcdcError,
    Plan,
    ccdc_plan,
    ccdc_plan_compression,
    ccdc_plan_jobs,
    ccdc_plan_jobs_repeated,
    load_library,
)
