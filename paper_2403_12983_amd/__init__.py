"""MI355X-native OSSCAR layer solver: thin ctypes binding over libosscar.so (hand-written HIP, gfx950)."""
from .binding import (OSSCAR_BF16, OSSCAR_F32, OSSCAR_INIT_GIVEN, OSSCAR_INIT_MAGNITUDE, OSSCAR_SEARCH_ALWAYS_ACCEPT,
                      OSSCAR_SEARCH_EAGER, OSSCAR_SEARCH_EXACT_IN, OSSCAR_SEARCH_NO_LOOKAHEAD, OsscarError, Solver, lib_path, load_library, osscar_gram_static, EXPORTED_SYMBOLS)

__all__ = ["Solver", "OsscarError", "osscar_gram_static", "load_library", "lib_path", "EXPORTED_SYMBOLS", "OSSCAR_F32", "OSSCAR_BF16",
           "OSSCAR_INIT_MAGNITUDE", "OSSCAR_INIT_GIVEN", "OSSCAR_SEARCH_ALWAYS_ACCEPT", "OSSCAR_SEARCH_EAGER", "OSSCAR_SEARCH_NO_LOOKAHEAD", "OSSCAR_SEARCH_EXACT_IN"]
