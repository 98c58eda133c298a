"""The five benchmark shapes: a single image, a tiled image, two videos and a
tiny case, each a visual segment on its patch grid followed by a text prompt.

A prefix is a list of consecutive segments.  A visual segment holds
``n_planes`` planes (tiles of one image, or frames of a video) of
``grid_h x grid_w`` patch tokens, row-major inside a plane.  ``temporal`` says
whether neighbouring planes are neighbouring frames (video) or independent
tiles.  Shapes follow the vision-token counts the paper reports for its models
(256 tokens per tile or frame, budgets 1024-4096, blocks 256-1024; Sec. 4.1 and
Tab. 4).
"""
from dataclasses import dataclass, field
from typing import List, Tuple

TEXT = 0
VISUAL = 1


@dataclass(frozen=True)
class Segment:
    token_begin: int
    n_tokens: int
    kind: int              # TEXT or VISUAL
    grid_h: int = 0
    grid_w: int = 0
    n_planes: int = 0
    temporal: int = 0      # 1: planes are video frames, 0: independent tiles


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    chunk: int             # block size b of Alg. 1
    budget: int            # memory budget M of Alg. 1, slots per KV head
    segments: Tuple[Segment, ...] = field(default_factory=tuple)
    # 'plane': every plane draws its own smooth field; 'shared': one field for
    # all planes plus a slowly drifting per-plane offset (video)
    field_unit: str = "plane"

    @property
    def n_tokens(self) -> int:
        return sum(s.n_tokens for s in self.segments)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


def _prefix(gh: int, gw: int, planes: int, temporal: int, n_text: int) -> Tuple[Segment, ...]:
    nvis = gh * gw * planes
    return (
        Segment(0, nvis, VISUAL, gh, gw, planes, temporal),
        Segment(nvis, n_text, TEXT),
    )


WORKLOADS: List[Workload] = [
    Workload("tiny", 1, 4, 4, 64, 64, 128, _prefix(24, 24, 1, 0, 32), "plane"),
    Workload("single_image", 4, 32, 32, 128, 128, 256, _prefix(24, 24, 1, 0, 64), "plane"),
    Workload("tiled_image", 8, 28, 4, 128, 256, 512, _prefix(24, 24, 5, 0, 128), "plane"),
    Workload("video", 16, 28, 4, 128, 512, 1024, _prefix(14, 14, 32, 1, 128), "shared"),
    Workload("long_video", 32, 32, 8, 128, 1024, 2048, _prefix(16, 16, 64, 1, 256), "shared"),
]


def get_workload(name_or_index) -> Workload:
    if isinstance(name_or_index, int):
        return WORKLOADS[name_or_index]
    for w in WORKLOADS:
        if w.name == name_or_index:
            return w
    raise KeyError(name_or_index)


def chunk_ranges(n_tokens: int, chunk: int):
    """Consecutive (token_begin, n) blocks of size ``chunk``; the last is short."""
    out = []
    t = 0
    while t < n_tokens:
        n = min(chunk, n_tokens - t)
        out.append((t, n))
        t += n
    return out
