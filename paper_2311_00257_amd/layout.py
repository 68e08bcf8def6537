"""Placement of the model-state streams in HBM.

The step reads and writes 2k + 7 streams at the same element index at the same time.  Large device
allocations all start on 2 MiB boundaries, so element i of every stream sits at the same offset modulo
8 KiB, and on MI355X a wave's loads of one vector from each stream then queue up behind each other in
the memory system: the fused step runs 4-6 % slower for k = 8 and k = 16 than with the streams' bases
shifted against each other (measured over fixed allocations, shifting only the views: any shift that is
not a multiple of 8 KiB restores the rate, multiples of 8 KiB up to 256 KiB do not; with k = 1, four
streams, it makes no difference).  The kernels cannot repair this, because element i of every stream
must meet in one wave, so the owner of the buffers does: stream j starts ``j * STAGGER_BYTES`` into an
allocation of its own.  4 KiB keeps every stream aligned to a wave's piece (512 B of bf16, 1 KiB of
fp32), which the kernels' fast path wants, and alternates neighbouring streams between the two halves of
the 8 KiB period.

Plumbing only: torch supplies the memory; nothing here computes."""
from __future__ import annotations

STAGGER_BYTES = 4096


def staggered_empty(specs, stagger: int = STAGGER_BYTES, first_index: int = 0, device: str = "cuda"):
    """One tensor per (elements, dtype) in ``specs``: tensor j is a view that starts
    ``(first_index + j) * stagger`` bytes into a fresh allocation of its own (stagger 0: plain
    ``torch.empty``).  The views keep their allocations alive."""
    import torch

    out = []
    for j, (elements, dtype) in enumerate(specs):
        item = torch.empty(0, dtype=dtype).element_size()
        if stagger == 0:
            out.append(torch.empty(elements, dtype=dtype, device=device))
            continue
        assert stagger % 1024 == 0, "keep every stream on a wave-piece boundary"
        offset = (first_index + j) * stagger
        raw = torch.empty(elements * item + offset, dtype=torch.uint8, device=device)
        out.append(raw[offset:offset + elements * item].view(dtype))
    return out
