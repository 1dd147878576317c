"""Alg. 1 (pattern-kind analysis, Sec. 4.2) as a CPU tool: the examples the listing names, the reading that makes the
result independent of the order of the reads, and the kinds of the decoder layer's own steps, which are what justifies
the fusions this library applies by hand."""
import itertools
import os

import pytest

from paper_2311_02103_amd import pattern_kind as pk

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "pattern_kind_examples.txt")


def golden_cases():
    with open(GOLDEN) as f:
        return [tuple(part.strip() for part in line.rsplit("=>", 1)) for line in f if line.strip() and not line.startswith("#")]


@pytest.mark.parametrize("program,kind", golden_cases())
def test_examples_named_by_the_listing(program, kind):
    assert kind in pk.KINDS
    assert pk.pattern_kind(program) == kind


def test_read_and_write_indices_of_the_listing_example():
    prog = pk.parse("C[i,j] = A[i,j] + B[j]")
    assert prog.read_tuples == [("i", "j"), ("j",)]
    assert prog.write_tuples == [("i", "j")]


def test_index_predicates():
    w = ("i", "j", "k")
    assert pk.is_element_wise(("i", "j", "k"), w) and not pk.is_element_wise(("i", "k", "j"), w)
    assert pk.is_broadcast(("j",), w) and pk.is_broadcast(("i", "k"), w)
    assert not pk.is_broadcast(("k", "i"), w)                 # order matters: that is a transpose, hence injective
    assert not pk.is_broadcast(("i", "j", "k"), w)            # proper sub-sequence only
    assert not pk.is_broadcast(("j//2",), w)                  # not a plain variable
    assert pk.is_injective(("k", "i"), w, set()) and pk.is_injective(("j//2", "(i+1)%4"), w, set())
    assert not pk.is_injective(("i", "r"), w, set())          # r is a reduction variable
    assert pk.is_injective(("T[i]", "N"), w, {"T"})           # tensors and size constants are not loop variables


def test_result_does_not_depend_on_the_order_of_the_reads():
    terms = ["A[i,j]", "B[j]", "D[j,i]", "E[i]"]
    kinds = {pk.pattern_kind("C[i,j] = " + " + ".join(p)) for p in itertools.permutations(terms)}
    assert kinds == {pk.INJECTIVE}
    kinds = {pk.pattern_kind("C[i,j] = " + " + ".join(p)) for p in itertools.permutations(terms[:2] + terms[3:])}
    assert kinds == {pk.ELEMENT_WISE}                          # broadcasts next to an element-wise read
    assert pk.pattern_kind("C[i,j] = B[j] * E[i]") == pk.BROADCAST


def test_a_bias_read_does_not_hide_a_matmul():
    assert pk.pattern_kind("C[i,j] += A[i,k] * B[k,j] * G[j]") == pk.OUT_EWISE_FUSIBLE
    assert pk.pattern_kind("C[i,j] += A[i,k] + B[k,j]") == pk.REDUCTION          # a sum over k of a sum: no multiply-add


def test_parse_errors():
    for bad in ("", "x = 1", "C[i,j A[i]", "C[i] <- A[i]"):
        with pytest.raises(ValueError):
            pk.pattern_kind(bad)


def test_kinds_of_the_decoder_layer_steps():
    for name, (program, kind) in pk.HOT_PATH_PROGRAMS.items():
        assert pk.pattern_kind(program) == kind, name


def test_hand_made_fusions_follow_the_kinds():
    kind = {name: pk.pattern_kind(src) for name, (src, _) in pk.HOT_PATH_PROGRAMS.items()}
    light = (pk.ELEMENT_WISE, pk.BROADCAST, pk.INJECTIVE)
    # the int4 decode is injective, so it may be inlined into its consumer; the fused program is still a multiply-add whose
    # output may take element-wise followers: that is the decode-in-matmul kernel with its epilogues
    assert kind["decode_q4"] == pk.INJECTIVE and kind["matmul"] == pk.OUT_EWISE_FUSIBLE
    assert kind["decode_q4_matmul"] == pk.OUT_EWISE_FUSIBLE
    for epilogue in ("rotary", "kv_append", "residual_add", "swiglu"):
        assert kind[epilogue] in light, epilogue
    # RMSNorm splits into a reduction-like pass and an element-wise scale: the scale is what rides in a matmul's prologue
    # (or in the finishing pass of the matmul before), the whole norm as one program could not be fused by kind
    assert kind["rms_scale"] == pk.ELEMENT_WISE and kind["rmsnorm_as_one_program"] == pk.OPAQUE
    # softmax as one program is opaque to the analysis: the attention kernels are written whole, not derived by fusion
    assert kind["softmax_as_one_program"] == pk.OPAQUE
    assert kind["attention_scores"] == kind["attention_values"] == pk.OUT_EWISE_FUSIBLE
    assert kind["row_max"] == pk.REDUCTION and kind["embedding_gather"] == pk.INJECTIVE
