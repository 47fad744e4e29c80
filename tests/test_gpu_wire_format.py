"""The boundary in the paper's wire format: packed q|k|v message in, 16-bit result out, one cache
allocation holding several layers (Sections 4.1.2, 4.3, 5.4.3)."""
import numpy as np
import pytest
import torch

from oracle import gh_oracle as O
from paper_2501_11779_amd import binding as G
from paper_2501_11779_amd import workloads as W
from tests import helpers as Hh

pytestmark = pytest.mark.gpu
DEV = "cuda"


round_f64_to_bits, ulps_apart = Hh.round_f64_to_bits, Hh.ulps_apart


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_rounding_helper_against_exactly_representable_and_midpoints(dtype):
    vals = np.array([0.0, 1.0, -1.0, 0.333251953125, 1.0 + 2.0 ** -9, 1.0 + 3 * 2.0 ** -9, 65504.0 / 4])
    bits = round_f64_to_bits(vals, dtype)
    back = W.from_bits(bits, dtype).double().numpy()
    step = 2.0 ** -10 if dtype == "f16" else 2.0 ** -7                 # spacing in [1, 2)
    assert back[0] == 0 and back[1] == 1 and back[2] == -1
    assert abs(back[3] - vals[3]) <= step / 2
    if dtype == "bf16":
        assert back[4] == 1.0                  # 1 + 2^-9 is below the midpoint 1 + 2^-8
        assert back[5] == 1.0 + 2.0 ** -7      # 1 + 3*2^-9 is above it
        mid = round_f64_to_bits(np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8]), dtype)
        assert W.from_bits(mid, dtype).double().tolist() == [1.0, 1.0 + 2.0 ** -6]   # ties to even


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("H,Hkv", [(8, 8), (16, 4)])
def test_packed_message_in_and_native_result_out(dtype, H, Hkv):
    lengths = np.array([0, 33, 200, 640, 64, 127], dtype=np.int32)
    B, d = len(lengths), 128
    w = W.Workload("wire", B, H, Hkv, d, dtype, ("const", 0), 81)
    inp = W.make_inputs(w, DEV, lengths=lengths, n_slots=B + 2)
    host = Hh.host_copy(inp)
    # one message per sequence: q (H*d) | k (H_kv*d) | v (H_kv*d), as Tier 1 would send it
    stride = (H + 2 * Hkv) * d
    msg = torch.cat([inp["q"].reshape(B, -1), inp["k_new"].reshape(B, -1),
                     inp["v_new"].reshape(B, -1)], dim=1).contiguous()
    assert msg.shape == (B, stride)
    e = msg.element_size()
    q_ptr = msg.data_ptr()
    k_ptr = q_ptr + H * d * e
    v_ptr = k_ptr + Hkv * d * e
    p = G.problem_from_inputs(inp)
    p.q_batch_stride = stride
    p.new_batch_stride = stride
    ws = G.alloc_workspace(p, DEV)
    ws.fill_(float("nan"))
    out16 = torch.full((B, H, d), float("nan"), dtype=W.TORCH_DTYPE[dtype], device=DEV)
    out32 = torch.full((B, H, d), float("nan"), dtype=torch.float32, device=DEV)
    G.check(G.gh_kv_append(p, inp["k_cache"], inp["v_cache"], k_ptr, v_ptr, inp["slot_id"],
                           inp["pos"], None))
    G.check(G.gh_decode_attention(p, q_ptr, inp["k_cache"], inp["v_cache"], inp["slot_id"],
                                  inp["ctx_len"], ws))
    G.check(G.gh_decode_reduce_native(p, ws, inp["ctx_len"], out16))
    G.check(G.gh_decode_reduce(p, ws, inp["ctx_len"], out32))
    torch.cuda.synchronize()

    want = Hh.oracle_step(inp, host)
    Hh.assert_parity(out32.cpu().numpy(), want, "packed message, fp32 result")
    assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])       # appended from the message
    assert np.array_equal(W.bits(inp["v_cache"]), host["v_cache"])
    # 16-bit result: the oracle rounded once to the same type; the fp32 path may land on the other
    # side of a rounding border for a few values, never further than one representable value
    got_bits = W.bits(out16)
    want_bits = round_f64_to_bits(want, dtype)
    apart = ulps_apart(got_bits, want_bits)
    # ... except next to zero, where one step of the 16-bit type is smaller than the fp32 path's
    # own absolute error (a few 1e-7) and the distance in steps means nothing
    far = apart > 1
    diff = np.abs(W.from_bits(got_bits, dtype).double().numpy() - W.from_bits(want_bits, dtype).double().numpy())
    assert np.all(diff[far] <= 2e-6)
    assert (apart == 0).mean() > 0.995
    # and it is exactly the fp32 result rounded to nearest even
    assert np.array_equal(got_bits, W.bits(out32.to(W.TORCH_DTYPE[dtype])))


def test_one_allocation_holding_several_layers():
    """Slots indexed by (layer, sequence): each layer's step gets that layer's base pointer."""
    n_layers, B, H, Hkv, d = 3, 4, 8, 2, 128
    lengths = np.array([100, 5, 300, 64], dtype=np.int32)
    layers = []
    for layer in range(n_layers):
        w = W.Workload(f"layer{layer}", B, H, Hkv, d, "bf16", ("const", 0), 90 + layer)
        layers.append(W.make_inputs(w, DEV, lengths=lengths, n_slots=B, capacity=320))
    k_all = torch.stack([x["k_cache"] for x in layers]).contiguous()     # [layer][slot][head][row][d]
    v_all = torch.stack([x["v_cache"] for x in layers]).contiguous()
    layer_bytes = k_all[0].numel() * k_all.element_size()
    hosts = [Hh.host_copy(x) for x in layers]
    out = torch.empty((B, H, d), dtype=torch.float32, device=DEV)
    for layer in reversed(range(n_layers)):                              # later layers first
        inp = layers[layer]
        p = G.problem_from_inputs(inp)
        ws = G.alloc_workspace(p, DEV)
        kb, vb = k_all.data_ptr() + layer * layer_bytes, v_all.data_ptr() + layer * layer_bytes
        G.check(G.gh_kv_append(p, kb, vb, inp["k_new"], inp["v_new"], inp["slot_id"], inp["pos"], None))
        G.check(G.gh_decode_attention(p, inp["q"], kb, vb, inp["slot_id"], inp["ctx_len"], ws))
        G.check(G.gh_decode_reduce(p, ws, None, out))
        torch.cuda.synchronize()
        Hh.assert_parity(out.cpu().numpy(), Hh.oracle_step(inp, hosts[layer]), f"layer {layer}")
    for layer in range(n_layers):                                        # no layer touched another
        assert np.array_equal(W.bits(k_all[layer]), hosts[layer]["k_cache"])
        assert np.array_equal(W.bits(v_all[layer]), hosts[layer]["v_cache"])


def test_batches_at_different_layers_merged_into_one_launch():
    """A Tier-2 node holds several batches in flight, each waiting at its own layer (Section 3.3).
    With the layers in one allocation their steps need not be launched one by one: the entries of
    all of them form one batch whose slot ids are layer * slots_per_layer + slot.  One launch of
    three 4-sequence batches must give each batch the result of its own step."""
    n_layers, B, H, Hkv, d = 3, 4, 8, 2, 128
    lengths = [np.array([100, 5, 300, 64], dtype=np.int32), np.array([0, 31, 32, 257], dtype=np.int32),
               np.array([319, 1, 77, 200], dtype=np.int32)]
    layers = []
    for layer in range(n_layers):
        w = W.Workload(f"inflight{layer}", B, H, Hkv, d, "bf16", ("const", 0), 95 + layer)
        layers.append(W.make_inputs(w, DEV, lengths=lengths[layer], n_slots=B, capacity=320))
    hosts = [Hh.host_copy(x) for x in layers]
    k_all = torch.stack([x["k_cache"] for x in layers]).contiguous()     # [layer][slot][head][row][d]
    v_all = torch.stack([x["v_cache"] for x in layers]).contiguous()
    cat = lambda name: torch.cat([x[name] for x in layers]).contiguous()
    merged = {"q": cat("q"), "k_new": cat("k_new"), "v_new": cat("v_new"), "pos": cat("pos"),
              "ctx_len": cat("ctx_len"), "k_cache": k_all, "v_cache": v_all,
              "slot_id": torch.cat([x["slot_id"] + layer * B for layer, x in enumerate(layers)])}
    p = G.make_problem(n_layers * B, H, Hkv, d, G.GH_BF16, n_layers * B, 320, 320,
                       layers[0]["strides"], layers[0]["scale"])
    ws = G.alloc_workspace(p, DEV)
    ws.fill_(float("nan"))
    out = torch.full((n_layers * B, H, d), float("nan"), dtype=torch.float32, device=DEV)
    G.decode_step(p, merged, ws, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    for layer in range(n_layers):
        Hh.assert_parity(got[layer * B:(layer + 1) * B], Hh.oracle_step(layers[layer], hosts[layer]),
                         f"batch at layer {layer}")
        assert np.array_equal(W.bits(k_all[layer]), hosts[layer]["k_cache"])
        assert np.array_equal(W.bits(v_all[layer]), hosts[layer]["v_cache"])
