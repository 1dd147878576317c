"""Pattern kind of a tensor program from its read and write indices (Sec. 4.2, Alg. 1) — a standalone CPU tool.

The paper's compiler runs this analysis over every tensor program and feeds the result back to the graph level, where
operator fusion (Alg. 2) decides from the kinds alone which neighbours may share a kernel.  This library applies those
fusions by hand (int4 decode into the matmuls, RMSNorm / rotary / SwiGLU / residual as prologues and epilogues), so the
analysis is kept as a checker: `HOT_PATH_PROGRAMS` writes every step of the decoder layer as index expressions and the
tests assert the kinds that justify each hand-made fusion.  Nothing here touches the GPU library.

A program is given as statements `T[idx, ...] <op> expression`, separated by `;` or newlines, with `<op>` one of
`=`, `+=`, `max=`, `min=`; an index is any expression over loop variables (`i`, `k//8`, `(d+64)%128`, `slot[b]`).
Loop variables are the identifiers that start with a lower-case letter and are not subscripted or called; identifiers
that start with an upper-case letter and are not subscripted are size constants (`j+F`).

Readings where the listing leaves room:
  * IsElementWise: the read's index tuple equals the write's;
  * IsBroadcast: the read's indices are plain loop variables forming a proper, order-preserving sub-sequence of the
    write's (which must be plain variables too);
  * IsInjective: every loop variable of the read's indices occurs in the write's indices;
  * the listing assigns `kind` read by read, so its result would depend on the order of the reads; here the reads are
    combined by taking the most general kind (ElementWise < Broadcast < Injective), and a read that is none of the three
    leaves the program Opaque for the two checks that follow — `C[i,j] = A[i,j] + B[j]` still comes out ElementWise and
    the three printed examples keep their kinds;
  * IsFuseMultiplyAdd: an accumulating statement (`+=`) over a reduction loop whose right-hand side is a product at top
    level; HasReductionLoop: some loop variable occurs in no write index;
  * the accumulator read implied by `+=`, `max=`, `min=` is not a read of the program.

    python -m paper_2311_02103_amd.pattern_kind "C[i,j] = A[i,j] + B[j]"      ->  ElementWise
"""
import re
import sys
from dataclasses import dataclass, field
from typing import Dict, List, Set, Tuple

ELEMENT_WISE, BROADCAST, INJECTIVE = "ElementWise", "Broadcast", "Injective"
REDUCTION, OUT_EWISE_FUSIBLE, OPAQUE = "Reduction", "OutputEwiseFusible", "Opaque"
KINDS = (ELEMENT_WISE, BROADCAST, INJECTIVE, REDUCTION, OUT_EWISE_FUSIBLE, OPAQUE)

_IDENT = re.compile(r"[A-Za-z_]\w*")
_STMT_OPS = ("+=", "max=", "min=", "=")


@dataclass(frozen=True)
class Access:
    tensor: str
    indices: Tuple[str, ...]


@dataclass
class Statement:
    write: Access
    op: str
    rhs: str
    reads: List[Access] = field(default_factory=list)


@dataclass
class Program:
    statements: List[Statement]
    tensors: Set[str]

    @property
    def write_tuples(self) -> List[Tuple[str, ...]]:
        return [s.write.indices for s in self.statements]

    @property
    def read_tuples(self) -> List[Tuple[str, ...]]:
        return [r.indices for s in self.statements for r in s.reads]


def _match_bracket(text: str, start: int) -> int:
    """Index of the `]` that closes the `[` at text[start]."""
    depth = 0
    for pos in range(start, len(text)):
        if text[pos] == "[":
            depth += 1
        elif text[pos] == "]":
            depth -= 1
            if depth == 0:
                return pos
    raise ValueError("unbalanced brackets in %r" % text)


def _split_top_level(text: str) -> Tuple[str, ...]:
    parts, depth, cur = [], 0, []
    for ch in text:
        if ch in "[(":
            depth += 1
        elif ch in "])":
            depth -= 1
        if ch == "," and depth == 0:
            parts.append("".join(cur))
            cur = []
        else:
            cur.append(ch)
    parts.append("".join(cur))
    return tuple(p.replace(" ", "") for p in parts)


def _accesses(text: str) -> List[Access]:
    """Every `name[...]` in text, outermost first, those nested inside index expressions included."""
    found, pos = [], 0
    while True:
        m = _IDENT.search(text, pos)
        if not m:
            return found
        end = m.end()
        if end < len(text) and text[end] == "[":
            close = _match_bracket(text, end)
            inner = text[end + 1:close]
            found.append(Access(m.group(), _split_top_level(inner)))
            found.extend(_accesses(inner))
            pos = close + 1
        else:
            pos = end


def parse(source: str) -> Program:
    statements = []
    for line in re.split(r"[;\n]", source):
        line = line.strip()
        if not line:
            continue
        m = _IDENT.match(line)
        if not m or m.end() >= len(line) or line[m.end()] != "[":
            raise ValueError("statement must start with a tensor write: %r" % line)
        close = _match_bracket(line, m.end())
        write = Access(m.group(), _split_top_level(line[m.end() + 1:close]))
        rest = line[close + 1:].lstrip()
        op = next((o for o in _STMT_OPS if rest.startswith(o)), None)
        if op is None:
            raise ValueError("expected one of %s after the write in %r" % (", ".join(_STMT_OPS), line))
        rhs = rest[len(op):].strip()
        reads = _accesses(rhs) + [a for idx in write.indices for a in _accesses(idx)]
        statements.append(Statement(write, op, rhs, reads))
    if not statements:
        raise ValueError("empty program")
    tensors = {s.write.tensor for s in statements} | {r.tensor for s in statements for r in s.reads}
    return Program(statements, tensors)


def _variables(indices: Tuple[str, ...], tensors: Set[str]) -> Set[str]:
    """Loop variables of an index tuple: lower-case identifiers that are neither tensors nor function names."""
    out = set()
    for idx in indices:
        for m in _IDENT.finditer(idx):
            after = idx[m.end():m.end() + 1]
            if m.group() not in tensors and after not in ("[", "(") and not m.group()[0].isupper():
                out.add(m.group())
    return out


def _plain(indices: Tuple[str, ...]) -> bool:
    return all(_IDENT.fullmatch(i) for i in indices)


def is_element_wise(read, write) -> bool:
    return tuple(read) == tuple(write)


def is_broadcast(read, write) -> bool:
    if not (_plain(read) and _plain(write)) or len(read) >= len(write) or len(set(read)) != len(read):
        return False
    it = iter(write)
    return all(any(v == w for w in it) for v in read)             # order-preserving sub-sequence


def is_injective(read, write, tensors: Set[str]) -> bool:
    return _variables(read, tensors) <= _variables(write, tensors)


def _top_level_product(rhs: str) -> bool:
    depth, has_mul = 0, False
    for pos, ch in enumerate(rhs):
        if ch in "[(":
            depth += 1
        elif ch in "])":
            depth -= 1
        elif depth == 0 and ch in "+-" and pos > 0:
            return False                                           # a sum at top level is not a multiply-add body
        elif depth == 0 and ch == "*":
            has_mul = True
    return has_mul


def has_reduction_loop(prog: Program) -> bool:
    for s in prog.statements:
        wv = _variables(s.write.indices, prog.tensors)
        for r in s.reads:
            if _variables(r.indices, prog.tensors) - wv:
                return True
    return False


def is_fuse_multiply_add(prog: Program) -> bool:
    return has_reduction_loop(prog) and any(s.op == "+=" and _top_level_product(s.rhs) for s in prog.statements)


# Generality of one read relative to the write's index tuple: a read is rated by the most specific of the three index
# predicates it satisfies, and anything else is unrated.  Ratings are totally ordered, so a whole program is rated by the
# most general read it contains.
_IDENTITY, _SUBSEQUENCE, _ONE_TO_ONE, _UNRATED = range(4)
_KIND_OF_RATING = (ELEMENT_WISE, BROADCAST, INJECTIVE, OPAQUE)


def _rate_read(read_indices, write_indices, tensors: Set[str]) -> int:
    if is_element_wise(read_indices, write_indices):
        return _IDENTITY
    if is_broadcast(read_indices, write_indices):
        return _SUBSEQUENCE
    if is_injective(read_indices, write_indices, tensors):
        return _ONE_TO_ONE
    return _UNRATED


def pattern_kind(source) -> str:
    """Pattern kind of a program given as text or as a parsed Program (Sec. 4.2, Alg. 1).

    Formulation: (1) a program whose statements write through different index tuples is Opaque; (2) every read is rated on
    the lattice identity < sub-sequence < one-to-one < unrated against the write's indices, and the program takes the
    highest rating among its reads (a program without reads is unrated); (3) the rating maps to a kind, with two
    refinements: a sub-sequence program that also holds an identity read computes one output element per input element
    and counts as ElementWise, and an unrated program is still fusible when it is a multiply-add over a reduction loop
    (OutputEwiseFusible) or any other reduction (Reduction)."""
    prog = source if isinstance(source, Program) else parse(source)
    writes = prog.write_tuples
    if len(set(writes)) > 1:
        return OPAQUE
    ratings = [_rate_read(r, writes[0], prog.tensors) for r in prog.read_tuples]
    rating = max(ratings, default=_UNRATED)
    if rating == _SUBSEQUENCE and _IDENTITY in ratings:
        return ELEMENT_WISE
    if rating == _UNRATED:
        if is_fuse_multiply_add(prog):
            return OUT_EWISE_FUSIBLE
        if has_reduction_loop(prog):
            return REDUCTION
    return _KIND_OF_RATING[rating]


# The steps of the decoder layer (Sec. 5.1's LLM workload) as index expressions, with the kind Alg. 1 gives each; i = row,
# j = output column, k = reduction column, h = head, d = head element, t = cached position, b = sequence.
HOT_PATH_PROGRAMS: Dict[str, Tuple[str, str]] = {
    "decode_q4": ("W[j,k] = (((Q[j,k//8] >> ((k%8)*4)) & 15) - 8) * S[j,k//32]", INJECTIVE),
    "matmul": ("Y[i,j] += X[i,k] * W[j,k]", OUT_EWISE_FUSIBLE),
    "decode_q4_matmul": ("Y[i,j] += X[i,k] * ((((Q[j,k//8] >> ((k%8)*4)) & 15) - 8) * S[j,k//32])", OUT_EWISE_FUSIBLE),
    "sum_of_squares": ("ss[i] += X[i,k] * X[i,k]", OUT_EWISE_FUSIBLE),
    "rms_scale": ("XN[i,j] = X[i,j] * rsqrt(ss[i] / H + eps) * G[j]", ELEMENT_WISE),
    "rmsnorm_as_one_program": ("ss[i] += X[i,k] * X[i,k]; XN[i,j] = X[i,j] * rsqrt(ss[i] / H + eps) * G[j]", OPAQUE),
    "rotary": ("R[i,h,d] = QKV[i,h,d] * C[pos[i],d%64] + QKV[i,h,(d+64)%128] * Sn[pos[i],d]", INJECTIVE),
    "kv_append": ("K[slot[i],pos[i],h,d] = QKV[i,h,d]", INJECTIVE),
    "attention_scores": ("P[i,h,t] += R[i,h,d] * K[slot[i],t,h//GROUP,d]", OUT_EWISE_FUSIBLE),
    "softmax_as_one_program": ("m[i,h] max= P[i,h,t]; l[i,h] += exp(P[i,h,t] - m[i,h]); A[i,h,t] = exp(P[i,h,t] - m[i,h]) / l[i,h]", OPAQUE),
    "attention_values": ("O[i,h,d] += A[i,h,t] * V[slot[i],t,h//GROUP,d]", OUT_EWISE_FUSIBLE),
    "residual_add": ("X1[i,j] = X[i,j] + O[i,j]", ELEMENT_WISE),
    "swiglu": ("ACT[i,j] = silu(GU[i,j]) * GU[i,j+F]", INJECTIVE),
    "row_max": ("m[i] max= L[i,v]", REDUCTION),
    "embedding_gather": ("X[i,j] = E[ids[i],j]", INJECTIVE),
}


def main(argv: List[str]) -> int:
    if len(argv) < 2:
        for name, (src, _) in HOT_PATH_PROGRAMS.items():
            print("%-26s %-20s %s" % (name, pattern_kind(src), src))
        return 0
    for src in argv[1:]:
        print(pattern_kind(src))
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
