"""Barnes-Hut t-SNE gradient step for MI355X (gfx950): thin binding over libtsne_hip.so."""
from .binding import (TsneParams, Tsne, build_P, build_P_workspace_bytes, lib, TsneError,  # noqa: F401
                      ivf_train, ivf_knn, build_P_approx, ivfpq_train, ivfpq_knn, kl_static,
                      STATUS_NONFINITE, STATUS_CELL_OVERFLOW, STATUS_WALK_OVERFLOW)
