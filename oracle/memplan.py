"""Plain reference for dynamic shape-aware memory planning (Relax, Sec. 4.3, Algorithm 3).

TEST INFRASTRUCTURE ONLY, like the rest of ``oracle/``: the product path never imports this module.

A program is a list of operations in execution order, each either

    ("alloc", tensor_name, size)       a tensor allocation, or
    ("call",  op_name, [tensor_names]) an operation that uses (reads or writes) the named tensors;

``outputs`` names the tensors that are still needed when the function returns (they are never dead).
A size is symbolic: ``("rows", c)`` stands for c * n bytes with n the symbolic row count, ``("opaque", k)`` for the k-th
expression the planner cannot decompose.  The steps are those of the algorithm, in its order:

  1. liveness analysis: the last operation that uses each tensor;
  2. a storage pool with symbolic-shape awareness, empty at first;
  3. walk the operations: an allocation asks the pool for a reusable storage and opens a new one when there is none;
     any other operation gives back the storage of every tensor it uses that is dead after it.

Two reuse rules:
  rule="equal"  the algorithm as Sec. 4.3 states it: a free storage is reused when the request's symbolic size is
                proven EQUAL to the storage's (the same multiple of n, the same opaque expression);
  rule="fits"   the extension the library lays its workspace out with (default here, because that is what the
                library's plan is compared with): the request only has to fit provably whatever the symbols are --
                equal expressions, or c1 * n into c2 * n with c1 <= c2 -- and the smallest such storage is taken.

The result maps every tensor to a storage index and every storage to the size expression it was opened with.
Pinned by tests/test_memplan.py (the four-tensors-into-two-chunks example of the paper's figure under both rules, cases
on which the rules differ, best fit, a brute force over all assignments on small programs, the no-overlap invariant,
and closed forms of the byte count).
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

Size = Tuple[str, int]


def provably_fits(want: Size, have: Size) -> bool:
    """True when a tensor of size `want` fits a storage opened for `have` for every value of the symbols."""
    if want[0] == "rows" and have[0] == "rows":
        return want[1] <= have[1]
    if want[0] == "opaque" and have[0] == "opaque":
        return want[1] == have[1]
    return False


def provably_equal(want: Size, have: Size) -> bool:
    """True when the two symbolic sizes are the same expression (the reuse condition of Sec. 4.3)."""
    return want[0] == have[0] and want[1] == have[1]


def liveness(program: Sequence[tuple], outputs: Sequence[str] = ()) -> Dict[str, int]:
    """Index of the last operation that uses each tensor (len(program) for the function's outputs)."""
    last: Dict[str, int] = {}
    for idx, op in enumerate(program):
        if op[0] == "alloc":
            last.setdefault(op[1], idx)
        else:
            for t in op[2]:
                last[t] = idx
    for t in outputs:
        last[t] = len(program)
    return last


def plan(program: Sequence[tuple], outputs: Sequence[str] = (), rule: str = "fits"):
    """Returns (storage_of_tensor: dict name -> storage index, storage_sizes: list of Size)."""
    assert rule in ("fits", "equal")
    reusable = provably_fits if rule == "fits" else provably_equal
    last = liveness(program, outputs)
    storage_sizes: List[Size] = []
    free: List[int] = []
    storage_of: Dict[str, int] = {}
    for idx, op in enumerate(program):
        if op[0] == "alloc":
            _, name, size = op
            candidates = [s for s in free if reusable(size, storage_sizes[s])]
            if candidates:
                # smallest storage that holds the request; sizes of one kind compare by their coefficient, and storages
                # of the other kind never are candidates
                s = min(candidates, key=lambda c: (storage_sizes[c][1], c))
                free.remove(s)
            else:
                s = len(storage_sizes)
                storage_sizes.append(size)
            storage_of[name] = s
            if last[name] == idx:                       # allocated and never used: dead at once
                free.append(s)
        else:
            for t in dict.fromkeys(op[2]):              # each tensor once, in the order it is named
                if last[t] == idx:
                    free.append(storage_of[t])
    return storage_of, storage_sizes


def evaluate(size: Size, n: int, opaque_bytes: Dict[int, int]) -> int:
    return size[1] * n if size[0] == "rows" else opaque_bytes[size[1]]


def planned_bytes(storage_sizes: Sequence[Size], n: int, opaque_bytes: Dict[int, int], align: int = 256) -> int:
    return sum((evaluate(s, n, opaque_bytes) + align - 1) // align * align for s in storage_sizes)
