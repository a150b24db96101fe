"""pbdr_render_fwd_static (the forward render on the library's own fixed scratch array, for callers that cannot
allocate) against pbdr_render_fwd with a caller workspace: bit for bit, on two calls in a row, the second smaller."""
import numpy as np
import pytest
import torch

from paper_2512_20017_amd import binding as B
from paper_2512_20017_amd import synth

pytestmark = pytest.mark.gpu


def _render_both(n, w, h, seed, bg):
    sc = synth.scene_tiny(seed, n=n)
    cam = synth.camera_tiny(w, h)
    scene = B.Scene.from_numpy(sc)
    splats = B.Splats.empty(n)
    B.pbdr_preprocess(scene, cam, splats)
    cap = B.PBDR_STATIC_MAX_PAIRS
    ws = B.alloc_workspace(n, w, h, cap)

    def outputs():
        return (torch.full((3, h, w), -7.0, device="cuda"), torch.full((h, w), -7.0, device="cuda"),
                torch.full((h, w), -7, dtype=torch.int32, device="cuda"))

    ref = outputs()
    B.pbdr_render_fwd(splats, cam, bg, cap, *ref, ws)
    pairs_ref, over = B.pbdr_query_lists(ws, n, w, h, cap)
    assert not over and pairs_ref > 0
    got = outputs()
    pair_count = torch.full((1,), 0xFFFFFFFF, dtype=torch.int64, device="cuda").to(torch.uint32)
    B.pbdr_render_fwd_static(splats, cam, bg, *got, pair_count)
    torch.cuda.synchronize()
    return ref, got, pairs_ref, int(pair_count.cpu().numpy()[0])


def test_static_scratch_forward_equals_workspace_forward_twice_second_smaller():
    # first call: several sort blocks, ragged image (not a multiple of the tile); second: fewer points, smaller image,
    # so the array still holds the first call's lists, ranges and counts behind and around what the second one uses
    for n, w, h, seed, bg in ((12000, 400, 296, 1, [0.1, 0.2, 0.3]), (700, 96, 80, 2, [0.0, 0.0, 0.0])):
        ref, got, pairs_ref, pairs_got = _render_both(n, w, h, seed, bg)
        assert pairs_got == pairs_ref
        for name, a, b in zip(("image", "final_T", "last_idx"), ref, got):
            assert torch.equal(a, b), (name, n, w, h)
        assert float(ref[1].min()) >= 0.0 and int(ref[2].max()) > 0      # the render did something
