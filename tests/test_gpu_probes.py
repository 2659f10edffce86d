"""GPU checks of the two machine probes the kernel designs lean on (include/cnnc.h, measurement aids): the issue rate of
a vector multiply-add by operand kind, and the cost of an LDS read by lane address pattern.  The assertions are the
qualitative facts the designs use, with wide margins; the numbers themselves are printed."""
import pytest

pytestmark = pytest.mark.gpu


def test_issue_rate_by_operand_kind():
    import paper_1508_01292_amd as P
    r = P.cnnc_measure_issue_rates()
    print("issue rates, ns per wave instruction and SIMD:", {k: round(v, 3) for k, v in r.items()}, flush=True)
    vec, lit = r["v_fmac_vector_operands"], r["v_fmac_literal_operand"]
    assert 0.5 < vec < 3.0
    assert lit < 1.25 * vec
    assert r["v_fmac_scalar_register_operand"] > 1.5 * lit          # why wave-uniform weights became literals
    assert r["v_rcp_f32"] > 2.0 * lit                               # the activation's reciprocal costs several slots


def test_lds_read_cost_by_pattern():
    import paper_1508_01292_amd as P
    L = P.cnnc_measure_lds_read
    lanes = range(64)
    t = {
        "b32 consecutive": L([i for i in lanes], 1),
        "b32 every second dword": L([2 * i for i in lanes], 1),                 # 32 banks, 32 lanes a pass: two-way conflict
        "b32 lanes l and l + 32 in one bank": L([(i % 32) + 64 * (i // 32) for i in lanes], 1),   # other half-wave: free
        "b64 consecutive": L([2 * i for i in lanes], 2),
        "b64 every second pair": L([4 * i for i in lanes], 2),                  # 64 banks, 32 lanes a pass: two-way conflict
        "b128 consecutive": L([4 * i for i in lanes], 4),
        "b128 every second quad": L([8 * i for i in lanes], 4),
        # lanes l and l + 4 read the same banks: free, because lanes 0-3 and 4-7 are served in different passes
        "b128 lanes l and l + 4 in the same banks": L([4 * (i % 4) + 64 * ((i // 4) % 2) + 16 * (i // 8) for i in lanes], 4),
        # lanes 0-3 and 12-15 are served together: the same banks there cost a pass
        "b128 lanes 0-3 and 12-15 in the same banks": L([(4 * (i % 4) + (64 if 12 <= i < 16 else 0)) if (i < 4 or 12 <= i < 16) else -1
                                                         for i in lanes], 4),
        "b128 lanes 0-3 and 4-7 in the same banks": L([(4 * (i % 4) + (64 if 4 <= i < 8 else 0)) if i < 8 else -1 for i in lanes], 4),
    }
    for k, v in t.items():
        print("%-46s %.3f ns per wave instruction and compute unit" % (k, v), flush=True)
    assert t["b32 every second dword"] > 1.4 * t["b32 consecutive"]
    assert t["b32 lanes l and l + 32 in one bank"] < 1.2 * t["b32 consecutive"]
    assert t["b64 consecutive"] < 1.3 * t["b32 consecutive"]                      # twice the bytes at the same cost
    assert t["b64 every second pair"] > 1.4 * t["b64 consecutive"]
    assert t["b128 every second quad"] > 1.6 * t["b128 consecutive"]
    assert t["b128 lanes l and l + 4 in the same banks"] < 1.2 * t["b128 consecutive"]
    assert t["b128 lanes 0-3 and 12-15 in the same banks"] > 1.1 * t["b128 lanes 0-3 and 4-7 in the same banks"]
    with pytest.raises(P.CnncError):
        L([0] * 64, 3)
    with pytest.raises(P.CnncError):
        L([2] * 64, 4)                    # not a multiple of the width
    with pytest.raises(P.CnncError):
        L([8708] * 64, 4)                 # outside the probe's array
