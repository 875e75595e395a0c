"""MI355X-native stage step and multi-ring parameter average (after Ravnest, arXiv 2401.01728)."""
from .api import (RV_BF16, RV_DECODER, RV_F32, RV_MLP, RvError, Stage, block_update, block_update_momentum,  # noqa: F401
                  cluster_average, cluster_sync, cluster_sync_fork, cluster_sync_join)
