"""MI355X-native implementation of ADORE's per-step decode path (arXiv 2407.02328).

`binding.Adore` wraps the C-ABI library libadore.so (HIP kernels for gfx950);
`build.build_library()` compiles it in-tree.
"""
from .binding import Adore, AdoreConfig, AdoreError, EXPORTS, KERNELS, LIB_PATH, load_library, make_config, topk_attention  # noqa: F401
