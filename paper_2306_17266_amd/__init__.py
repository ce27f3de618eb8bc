"""MI355X-native SubGraph-Stationary SubNet inference (arXiv 2306.17266): thin Python binding of the
HIP library libsushi.so.  Importing this package does not load the library; the first call does,
and it raises if the library has not been built — there is no CPU fallback."""
from .binding import (BF16, FP32, OPT_EXEC_MODE, OPT_KERNEL_TIMING, OPT_SPIN_LIMIT, OPT_IDLE_US, OPT_STREAM_WGS, OPT_TEAM_WGS_PER_CU, OPT_TEAMS_PER_XCD, OPT_COLD_SWEEP_MIB, OPT_PATCH_CONV_MIN_PIXELS, STRICT_ACCURACY, STRICT_LATENCY, Sushi, SushiError,  # noqa: F401
                      sushi_describe_supernet, sushi_pack_supernet, sushi_subgraph_overlap, sushi_subnet_layers, sushi_team_plan)
