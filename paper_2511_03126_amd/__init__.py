"""MI355X-native multi-view feature fusion, material scoring and property integration.

Thin Python front end of libaura_fuse.so (hand-written HIP for gfx950).  Nothing is computed in
Python: every function in `binding` marshals torch tensors into one C-ABI call.
"""
from . import binding  # noqa: F401
from .binding import (Params, Views, estimate_normals, fuse_features, fuse_score_integrate,  # noqa: F401
                      fuse_score_integrate_workspace_bytes, fuse_scores, fuse_scores_workspace_bytes, fuse_selected,
                      fuse_workspace_bytes, knn_densify, material_scores, material_scores_static, patch_batch,
                      project_visibility, property_integrate, select_views, thickness_integrate, time_next_fusion,
                      voxel_downsample, voxel_grid, voxel_workspace_bytes, workspace_bytes)
