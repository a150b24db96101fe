"""Run the HIP path through the C-ABI binding and hand back numpy arrays in the oracle's layouts (test helper)."""
import numpy as np
import torch

from paper_2512_20017_amd import binding as B


def to_hwc(img_chw: torch.Tensor) -> np.ndarray:
    return img_chw.permute(1, 2, 0).contiguous().cpu().numpy()


def to_chw_dev(img_hwc: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(np.asarray(img_hwc, dtype=np.float32).transpose(2, 0, 1))).cuda()


class GpuView:
    """One view's buffers: splats, workspace, image outputs, splat grads."""

    def __init__(self, n, cam, dup_capacity):
        self.n, self.cam, self.cap = n, cam, int(dup_capacity)
        W, H = cam["width"], cam["height"]
        self.W, self.H = W, H
        self.splats = B.Splats.empty(n)
        self.ws = B.alloc_workspace(n, W, H, self.cap)
        self.image = torch.empty((3, H, W), dtype=torch.float32, device="cuda")
        self.final_T = torch.empty((H, W), dtype=torch.float32, device="cuda")
        self.last_idx = torch.empty((H, W), dtype=torch.int32, device="cuda")
        self.g_splats = B.SplatGrads.empty(n)

    def preprocess(self, scene):
        B.pbdr_preprocess(scene, self.cam, self.splats)
        torch.cuda.synchronize()
        return self.splats.to_numpy()

    def render_fwd(self, bg, splats=None):
        sp = splats if splats is not None else self.splats
        B.pbdr_render_fwd(sp, self.cam, bg, self.cap, self.image, self.final_T, self.last_idx, self.ws)
        torch.cuda.synchronize()
        return dict(image=to_hwc(self.image), final_T=self.final_T.cpu().numpy(),
                    last_idx=self.last_idx.cpu().numpy().astype(np.uint32))

    def lists(self):
        return B.pbdr_lists_view(self.ws, self.n, self.W, self.H, self.cap)

    def render_bwd(self, bg, dL_dimage_hwc, scene=None, grads=None, splats=None):
        sp = splats if splats is not None else self.splats
        g = to_chw_dev(dL_dimage_hwc)
        B.pbdr_render_bwd(scene, sp, self.cam, bg, self.cap, self.final_T, self.last_idx, g, self.g_splats, grads, self.ws)
        torch.cuda.synchronize()
        return self.g_splats.to_numpy()


def num_pairs_upper_bound(oracle_mod, sp_np, W, H):
    """Exact pair count for the GPU's own splats, from the oracle's binning (used to size dup_capacity)."""
    lists = oracle_mod.bin_sort(sp_np["mean2d"].astype(np.float64), sp_np["radius"], sp_np["depth"], W, H)
    return lists["P"], lists
