"""MI355X-native schedule-executed training step (MONeT, arxiv 2010.14501): thin binding over libmonet.so."""
from .monet import (Plan, MonetError, EVENT_DTYPE, load_library, library_path,  # noqa: F401
                    ALLOC, FREE, RUN_FWD, RUN_RECOMPUTE, RUN_BWD, SAVE, ALIAS)
