"""Device placement of the draft model beside a pipeline-parallel target (paper, appendix on resource-constrained
scenarios).  Test infrastructure / design aid only: this build runs on one GPU and ships no multi-GPU code; the
function states which device each model occupies over one target forward so that the strategy can be checked
against the paper's worked example and for freedom from collisions.

Time is cut into g*c slots of equal length: the target (speed ratio c, pipeline of g devices) spends c slots on
each device in turn; the draft model needs g slots per draft token and produces gamma of them per target forward.
Its first ceil(gamma/2) tokens are produced on the last device, the remaining floor(gamma/2) on the first one.
"""
from typing import List, Tuple


def occupancy(c: int, g: int, gamma: int) -> Tuple[List[int], List[int]]:
    """(device of the target per slot, device of the draft model per slot; -1 = idle) over the g*c slots of one
    target forward."""
    if c < 1 or g < 2 or gamma < 1:
        raise ValueError("c >= 1, g >= 2 devices, gamma >= 1")
    slots = g * c
    target = [s // c for s in range(slots)]
    first = -(-gamma // 2)                       # tokens produced on the last device
    draft = []
    for tok in range(gamma):
        draft += [g - 1 if tok < first else 0] * g
    draft = (draft + [-1] * slots)[:max(slots, len(draft))]
    return target, draft


def collisions(c: int, g: int, gamma: int) -> int:
    """Slots of one target forward in which both models sit on the same device."""
    target, draft = occupancy(c, g, gamma)
    return sum(1 for s, dev in enumerate(target) if s < len(draft) and draft[s] == dev)
