"""The C-ABI library without a GPU: it loads, exports every declared symbol, and turns
every bad argument into its status code before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2505_07291_amd as grpo

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, NULL, SHAPE, DTYPE, ALIGN, PARAM, WORKSPACE, HIP, CAPACITY = range(9)
P = 0x7F0000001000  # a fake, 256-byte aligned, non-null "device pointer": validation never dereferences


def declared_functions():
    text = open(os.path.join(ROOT, "include", "grpo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(grpo_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"grpo_group_advantages", "grpo_logprobs_fwd", "grpo_loss_fwd_bwd", "grpo_loss_aux_fwd_bwd",
            "grpo_packed_layout", "grpo_total_rewards", "grpo_filter_groups",
            "grpo_workspace_bytes", "grpo_status_string", "grpo_workspace_error"} <= set(names)
    L = grpo.lib()
    for n in names:
        assert hasattr(L, n), n


def test_status_strings_and_workspace_size():
    for code in range(9):
        assert len(grpo.status_string(code)) > 1
    assert grpo.status_string(99) == "unknown status"
    assert grpo.grpo_workspace_bytes(-1) == 0
    assert grpo.grpo_workspace_bytes(0) >= 256 and grpo.grpo_workspace_bytes(0) % 256 == 0
    for n in (1, 255, 256, 257, 131072):
        b = grpo.grpo_workspace_bytes(n)
        assert b % 256 == 0 and b >= 256 + 13 * n


def test_row_kernel_plan_covers_every_width():
    """The host logic that picks a row kernel: every width gets a kernel that can hold or stream
    it, ragged rows only kernels that handle a ragged tail, and what is held fits the chip."""
    import ctypes
    from paper_2505_07291_amd.binding import RowPlan
    L = grpo.lib()
    out = RowPlan()
    assert L.grpo_row_kernel_plan(7, 1000, ctypes.byref(out)) == DTYPE
    assert L.grpo_row_kernel_plan(1, 0, ctypes.byref(out)) == SHAPE
    assert L.grpo_row_kernel_plan(1, (1 << 28) + 1, ctypes.byref(out)) == SHAPE
    assert L.grpo_row_kernel_plan(1, 1000, None) == NULL
    rng = np.random.default_rng(1)
    limits = [256, 1024, 4096, 6656, 8192, 10240, 13312, 16384, 19456, 22528, 27648, 30720, 34816, 67584]
    for dtype, epv in ((grpo.GRPO_BF16, 8), (grpo.GRPO_F32, 4)):
        vocabs = set(range(1, 70)) | {int(v) for v in np.exp(rng.uniform(0, np.log(2.0 ** 28), 400))} | {1 << 28}
        for lim in limits:                                      # both sides of every limit, ragged or not
            vocabs |= {lim * epv - 1, lim * epv, lim * epv + 1, lim * epv + epv}
        for vocab in sorted(vocabs):
            p = grpo.grpo_row_kernel_plan(dtype, vocab)
            nvec, ragged = (vocab + epv - 1) // epv, vocab % epv != 0
            assert p["vectors"] == nvec
            if p["streaming"]:
                assert p["resident_vectors"] == 0
                assert (ragged and nvec > 10240) or nvec > 67584, (dtype, vocab)
                continue
            cap = p["lanes"] * (p["register_slots"] + p["lds_slots"])
            assert p["resident_vectors"] == min(nvec, cap)
            if p["streamed_remainder"]:
                assert cap < nvec <= 2 * cap
            else:
                assert nvec <= cap, (dtype, vocab, p)
            assert not ragged or p["ragged_tail_slot"], (dtype, vocab, p)
            # what is held fits: 512 KB of registers and 160 KB of LDS per CU
            lanes_per_cu = p["lanes"] * p["workgroups_per_cu"]
            assert lanes_per_cu <= 2048
            assert p["register_slots"] * 16 * lanes_per_cu <= 432 * 1024
            assert p["lds_slots"] * 16 * lanes_per_cu <= 160 * 1024
    bench = grpo.grpo_row_kernel_plan(grpo.GRPO_BF16, 152064)
    assert (bench["lanes"], bench["register_slots"], bench["lds_slots"], bench["streaming"]) == (512, 38, 0, 0)
    assert bench["resident_vectors"] == bench["vectors"] == 19008
    wide = grpo.grpo_row_kernel_plan(grpo.GRPO_BF16, 262144)
    assert wide["lds_slots"] == 18 and wide["resident_vectors"] == wide["vectors"] and not wide["streamed_remainder"]
    f32 = grpo.grpo_row_kernel_plan(grpo.GRPO_F32, 152064)
    assert f32["streamed_remainder"] == 1 and f32["resident_vectors"] == 512 * 66 < f32["vectors"]
    assert grpo.grpo_row_kernel_plan(grpo.GRPO_BF16, 152069)["streaming"] == 1   # ragged and wide


def loss_args(**over):
    a = dict(logits=P, dtype=1, n=16, V=1024, stride=1024, tokens=P, old=P, adv=P, mask=P,
             el=0.2, eh=0.2, delta=4.0, T=1.0, denom=0.0, gs=1.0, loss=P, lp=P, counts=P, grad=P,
             ws=P, ws_bytes=1 << 20, stream=None)
    a.update(over)
    return [a[k] for k in ("logits", "dtype", "n", "V", "stride", "tokens", "old", "adv", "mask",
                           "el", "eh", "delta", "T", "denom", "gs", "loss", "lp", "counts", "grad",
                           "ws", "ws_bytes", "stream")]


@pytest.mark.parametrize("over,expect", [
    (dict(logits=None), NULL), (dict(tokens=None), NULL), (dict(old=None), NULL),
    (dict(adv=None), NULL), (dict(loss=None), NULL), (dict(grad=None), NULL),
    (dict(n=-1), SHAPE), (dict(V=0), SHAPE), (dict(stride=1000), SHAPE), (dict(V=(1 << 28) + 8, stride=(1 << 28) + 8), SHAPE),
    (dict(dtype=2), DTYPE), (dict(dtype=-1), DTYPE),
    (dict(logits=P + 8), ALIGN), (dict(grad=P + 2), ALIGN), (dict(V=1001, stride=1001), ALIGN),
    (dict(dtype=0, V=1001, stride=1002), ALIGN),
    (dict(T=0.0), PARAM), (dict(T=-1.0), PARAM), (dict(T=float("nan")), PARAM),
    (dict(el=-0.1), PARAM), (dict(el=1.5), PARAM), (dict(eh=-0.2), PARAM),
    (dict(delta=1.2), PARAM), (dict(delta=1.0), PARAM), (dict(delta=float("nan")), PARAM),
    (dict(eh=float("inf")), PARAM), (dict(denom=float("nan")), PARAM),
    (dict(ws=None), WORKSPACE), (dict(ws=P + 64), WORKSPACE), (dict(ws_bytes=100), WORKSPACE),
])
def test_loss_fwd_bwd_rejects_bad_arguments_before_any_launch(over, expect):
    assert grpo.lib().grpo_loss_fwd_bwd(*loss_args(**over)) == expect


def noalloc_args(**over):
    a = dict(logits=P, dtype=1, n=16, V=1024, stride=1024, tokens=P, old=P, adv=P, mask=P,
             el=0.2, eh=0.2, delta=4.0, T=1.0, denom=0.0, gs=1.0, loss=P, lp=P, counts=P, grad=P,
             err=P, stream=None)
    a.update(over)
    return [a[k] for k in ("logits", "dtype", "n", "V", "stride", "tokens", "old", "adv", "mask",
                           "el", "eh", "delta", "T", "denom", "gs", "loss", "lp", "counts", "grad",
                           "err", "stream")]


@pytest.mark.parametrize("over,expect", [
    (dict(n=grpo.NOALLOC_MAX_TOKENS + 1), CAPACITY), (dict(n=1 << 40), CAPACITY),
    (dict(logits=None), NULL), (dict(old=None), NULL), (dict(loss=None), NULL), (dict(grad=None), NULL),
    (dict(n=-1), SHAPE), (dict(V=0), SHAPE), (dict(stride=1000), SHAPE), (dict(dtype=2), DTYPE),
    (dict(logits=P + 8), ALIGN), (dict(grad=P + 2), ALIGN),
    (dict(T=0.0), PARAM), (dict(el=1.5), PARAM), (dict(delta=1.2), PARAM), (dict(denom=float("nan")), PARAM),
])
def test_noalloc_variant_rejects_bad_arguments_before_any_launch(over, expect):
    """The entry point without a workspace: the row limit of its built-in scratch array is checked
    first and by itself (no device is needed to refuse), then the same argument checks as the
    workspace variant."""
    assert grpo.lib().grpo_loss_fwd_bwd_noalloc(*noalloc_args(**over)) == expect
    assert "GRPO_NOALLOC_MAX_TOKENS" in grpo.status_string(CAPACITY)
    hdr = open(os.path.join(ROOT, "include", "grpo.h")).read()
    assert "#define GRPO_NOALLOC_MAX_TOKENS %d" % grpo.NOALLOC_MAX_TOKENS in hdr


def test_logprobs_and_advantages_reject_bad_arguments():
    L = grpo.lib()
    f = L.grpo_logprobs_fwd
    assert f(None, 1, 4, 64, 64, P, None, 1.0, P, None, 0, None) == NULL
    assert f(P, 1, 4, 64, 64, None, None, 1.0, P, None, 0, None) == NULL
    assert f(P, 1, 4, 64, 64, P, None, 1.0, None, None, 0, None) == NULL
    assert f(P, 1, 4, 64, 60, P, None, 1.0, P, None, 0, None) == SHAPE
    assert f(P, 3, 4, 64, 64, P, None, 1.0, P, None, 0, None) == DTYPE
    assert f(P + 4, 1, 4, 64, 64, P, None, 1.0, P, None, 0, None) == ALIGN
    assert f(P, 1, 4, 63, 63, P, None, 1.0, P, None, 0, None) == ALIGN     # 126-byte row pitch
    assert f(P, 1, 4, 64, 64, P, None, 0.0, P, None, 0, None) == PARAM
    assert f(P, 1, 4, 64, 64, P, None, 1.0, P, P + 8, 1 << 16, None) == WORKSPACE   # misaligned
    assert f(P, 1, 4, 64, 64, P, None, 1.0, P, P, 100, None) == WORKSPACE       # too small
    assert f(P, 1, 0, 64, 64, None, None, 1.0, None, None, 0, None) == OK   # nothing to do
    g = L.grpo_group_advantages
    assert g(None, 8, None, 2, 4, 1e-6, 0, P, None, 0, None, None) == NULL
    assert g(P, 8, None, 2, 4, 1e-6, 0, None, None, 0, None, None) == NULL
    assert g(P, 8, None, 2, 3, 1e-6, 0, P, None, 0, None, None) == SHAPE   # 2*3 != 8
    assert g(P, 8, None, 2, 0, 1e-6, 0, P, None, 0, None, None) == SHAPE
    assert g(P, -1, None, 2, 4, 1e-6, 0, P, None, 0, None, None) == SHAPE
    assert g(P, 8, None, 2, 4, -1.0, 0, P, None, 0, None, None) == PARAM
    assert g(P, 8, None, 2, 4, 1e-6, 2, P, None, 0, None, None) == PARAM
    assert g(P, 8, None, 2, 4, 1e-6, 0, P, P, 10, None, None) == NULL       # adv_tok_out missing
    assert g(P, 0, None, 0, 4, 1e-6, 0, None, None, 0, None, None) == OK    # nothing to do
    e = L.grpo_workspace_error
    flag = ctypes.c_int32(7)
    assert e(None, ctypes.byref(flag), None) == NULL
    assert e(P, None, None) == NULL


def test_binding_refuses_cpu_tensors():
    import torch
    z = torch.zeros(4, 64)
    with pytest.raises(ValueError):
        grpo.grpo_logprobs_fwd(z, torch.zeros(4, dtype=torch.int64))


def aux_args(**over):
    a = dict(logits=P, dtype=1, n=16, V=1024, stride=1024, tokens=P, old=P, ref=P, adv=P, mask=P, tw=None,
             el=0.2, eh=0.2, delta=4.0, T=1.0, klc=0.001, enc=1e-4, denom=0.0, gs=1.0, loss=P, lp=P,
             ent=P, counts=P, grad=P, ws=P, ws_bytes=1 << 20, stream=None)
    a.update(over)
    return [a[k] for k in ("logits", "dtype", "n", "V", "stride", "tokens", "old", "ref", "adv", "mask",
                           "tw", "el", "eh", "delta", "T", "klc", "enc", "denom", "gs", "loss", "lp", "ent",
                           "counts", "grad", "ws", "ws_bytes", "stream")]


@pytest.mark.parametrize("over,expect", [
    (dict(ref=None), NULL),                       # a KL term needs reference log-probs
    (dict(old=None), NULL), (dict(loss=None), NULL), (dict(grad=None), NULL),
    (dict(klc=float("nan")), PARAM), (dict(enc=float("inf")), PARAM), (dict(delta=1.1), PARAM),
    (dict(T=0.0), PARAM), (dict(V=0), SHAPE), (dict(dtype=7), DTYPE), (dict(logits=P + 2), ALIGN),
    (dict(ws_bytes=256 + 5 * 16), WORKSPACE), (dict(ws=None), WORKSPACE),
])
def test_loss_aux_rejects_bad_arguments_before_any_launch(over, expect):
    assert grpo.lib().grpo_loss_aux_fwd_bwd(*aux_args(**over)) == expect


def test_packed_layout_rejects_bad_arguments():
    f = grpo.lib().grpo_packed_layout
    assert f(None, 4, 100, 1, P, P, None) == NULL
    assert f(P, 4, 100, 1, None, None, None) == NULL
    assert f(P, -1, 100, 1, P, P, None) == SHAPE
    assert f(P, 4, -5, 0, P, P, None) == SHAPE
    assert f(P, 4, 0, 0, P, None, None) == OK                  # nothing to do


def test_reward_helpers_reject_bad_arguments():
    L = grpo.lib()
    f = L.grpo_total_rewards
    assert f(None, P, P, 8, 3e-4, P, None) == NULL
    assert f(P, P, P, 8, 3e-4, None, None) == NULL
    assert f(P, P, P, -1, 3e-4, P, None) == SHAPE
    assert f(P, P, P, 8, float("nan"), P, None) == PARAM
    assert f(None, None, None, 0, 3e-4, None, None) == OK
    h = L.grpo_filter_groups
    assert h(P, 8, None, 2, 4, P, P, None, None, None) == NULL       # n_kept_out missing
    assert h(P, 8, None, 2, 4, None, P, P, None, None) == NULL
    assert h(None, 8, None, 2, 4, P, P, P, None, None) == NULL
    assert h(P, 8, None, 2, 3, P, P, P, None, None) == SHAPE
    assert h(P, 8, None, -2, 4, P, P, P, None, None) == SHAPE


def lmhead_args(**over):
    a = dict(hidden=P, hs=128, weight=P, wstride=128, n=16, V=1000, d=128, tokens=P, old=P, adv=P, mask=P,
             el=0.2, eh=0.2, delta=4.0, T=1.0, denom=0.0, gs=1.0, loss=P, lp=P, counts=P,
             gh=P, ghs=128, gw=P, gws=128, acc=0, ws=P, ws_bytes=1 << 30, stream=None)
    a.update(over)
    return [a[k] for k in ("hidden", "hs", "weight", "wstride", "n", "V", "d", "tokens", "old", "adv",
                           "mask", "el", "eh", "delta", "T", "denom", "gs", "loss", "lp", "counts",
                           "gh", "ghs", "gw", "gws", "acc", "ws", "ws_bytes", "stream")]


@pytest.mark.parametrize("over,expect", [
    (dict(hidden=None), NULL), (dict(weight=None), NULL), (dict(tokens=None), NULL), (dict(old=None), NULL),
    (dict(adv=None), NULL), (dict(loss=None), NULL), (dict(gh=None), NULL), (dict(gw=None), NULL),
    (dict(n=-1), SHAPE), (dict(V=0), SHAPE), (dict(d=0), SHAPE), (dict(d=80, hs=80, wstride=80), SHAPE), (dict(d=96, hs=96, wstride=96), SHAPE),
    (dict(hs=64), SHAPE), (dict(wstride=120), SHAPE), (dict(ghs=64), SHAPE), (dict(gws=100), SHAPE),
    (dict(V=(1 << 28) + 1), SHAPE), (dict(d=1 << 21, hs=1 << 21, wstride=1 << 21), SHAPE),
    (dict(hidden=P + 8), ALIGN), (dict(weight=P + 2), ALIGN), (dict(hs=132), ALIGN), (dict(wstride=129), ALIGN),
    (dict(T=0.0), PARAM), (dict(T=float("nan")), PARAM), (dict(el=1.5), PARAM), (dict(eh=-0.1), PARAM),
    (dict(delta=1.2), PARAM), (dict(denom=float("nan")), PARAM),
    (dict(ws=None), WORKSPACE), (dict(ws=P + 64), WORKSPACE), (dict(ws_bytes=4096), WORKSPACE),
])
def test_lmhead_loss_rejects_bad_arguments_before_any_launch(over, expect):
    assert grpo.lib().grpo_lmhead_loss_fwd_bwd(*lmhead_args(**over)) == expect


def test_lmhead_logprobs_rejects_bad_arguments_and_sizes_its_workspace():
    L = grpo.lib()
    ok = dict(hidden=P, hs=128, weight=P, wstride=128, n=16, V=1000, d=128, tokens=P, mask=None, T=1.0,
              lp=P, ws=P, ws_bytes=1 << 30, stream=None)

    def call(**over):
        a = dict(ok)
        a.update(over)
        return L.grpo_lmhead_logprobs_fwd(*[a[k] for k in ("hidden", "hs", "weight", "wstride", "n", "V", "d",
                                                           "tokens", "mask", "T", "lp", "ws", "ws_bytes",
                                                           "stream")])
    assert call(n=0, hidden=None, tokens=None, lp=None) == OK     # nothing to do
    assert call(lp=None) == NULL and call(hidden=None) == NULL
    assert call(d=100, hs=100, wstride=100) == SHAPE and call(T=-1.0) == PARAM
    assert call(ws=None) == WORKSPACE and call(ws_bytes=64) == WORKSPACE
    assert call(hs=130) == ALIGN
    # workspace sizes: forward holds a compacted copy of the hidden states and 8 bytes per token
    # and 256 vocabulary entries; the backward works in chunks of rows and holds, per chunk row, the
    # logits (fp32) and their gradient (bf16): its size follows the chunk (10240 rows by default), not the
    # number of tokens, and no copy of the weights is part of it
    n, V, d = 16384, 152064, 5120
    fwd = grpo.grpo_lmhead_workspace_bytes(n, V, d, False)
    bwd = grpo.grpo_lmhead_workspace_bytes(n, V, d, True)
    assert fwd % 256 == 0 and bwd % 256 == 0
    assert fwd < 300 << 20 and fwd >= grpo.grpo_workspace_bytes(n) + 8 * n * ((V + 255) // 256) + 2 * n * d
    chunk = 10240
    assert bwd >= 6 * chunk * V and bwd < 7 * chunk * V + 64 * n + 8 * n * d
    assert bwd <= 4 * n * V + 4 * V * d                    # at most 4 bytes per logit of this batch
    by_chunk = grpo.grpo_lmhead_workspace_bytes_for_chunk
    assert by_chunk(n, V, d, chunk) == bwd and by_chunk(n, V, d, 10000) == bwd      # rounded up to 256 rows
    assert by_chunk(n, V, d, 256) < by_chunk(n, V, d, 512) < bwd < by_chunk(n, V, d, n) == by_chunk(n, V, d, 10 ** 9)
    big = grpo.grpo_lmhead_workspace_bytes(131072, V, d, True)                     # eight times the tokens:
    assert big - bwd < 64 * (131072 - n) + 2 * (131072 - n) * d + 4096             # only per-row arrays grow
    assert grpo.grpo_lmhead_workspace_bytes(300, V, d, True) == by_chunk(300, V, d, 512)   # fewer rows than a chunk
    assert grpo.grpo_lmhead_workspace_bytes(-1, V, d, True) == 0
    assert grpo.grpo_lmhead_workspace_bytes(n, 0, d, True) == 0
    assert by_chunk(n, V, d, 0) == 0 and by_chunk(n, V, 100, 256) == 0
    # with the backward the vocabulary is limited by 32-bit offsets inside an operand tile
    assert grpo.grpo_lmhead_workspace_bytes(16, 8388544, 64, True) > 0
    assert grpo.grpo_lmhead_workspace_bytes(16, 8388545, 64, True) == 0
    assert grpo.grpo_lmhead_workspace_bytes(16, 8388545, 64, False) > 0
    assert L.grpo_lmhead_loss_fwd_bwd(*lmhead_args(V=8388545, ws_bytes=1 << 60)) == SHAPE
    # a workspace below the 256-row size is refused, anything from there on is taken
    need = by_chunk(16, 1000, 128, 256)
    assert L.grpo_lmhead_loss_fwd_bwd(*lmhead_args(ws_bytes=need - 256)) == WORKSPACE


def lmhead_aux_args(**over):
    a = dict(hidden=P, hs=128, weight=P, wstride=128, n=16, V=1000, d=128, tokens=P, old=P, ref=P, adv=P,
             mask=P, tw=None, el=0.2, eh=0.2, delta=4.0, T=1.0, klc=0.001, enc=1e-4, denom=0.0, gs=1.0,
             loss=P, lp=P, ent=None, counts=P, gh=P, ghs=128, gw=P, gws=128, acc=0, ws=P, ws_bytes=1 << 30,
             stream=None)
    a.update(over)
    return [a[k] for k in ("hidden", "hs", "weight", "wstride", "n", "V", "d", "tokens", "old", "ref", "adv",
                           "mask", "tw", "el", "eh", "delta", "T", "klc", "enc", "denom", "gs", "loss", "lp",
                           "ent", "counts", "gh", "ghs", "gw", "gws", "acc", "ws", "ws_bytes", "stream")]


@pytest.mark.parametrize("over,expect", [
    (dict(hidden=None), NULL), (dict(old=None), NULL), (dict(loss=None), NULL), (dict(gw=None), NULL),
    (dict(ref=None), NULL),                       # a KL coefficient needs the reference log-probs
    (dict(n=-1), SHAPE), (dict(d=80, hs=80, wstride=80), SHAPE), (dict(d=96, hs=96, wstride=96), SHAPE), (dict(ghs=64), SHAPE),
    (dict(weight=P + 2), ALIGN),
    (dict(T=0.0), PARAM), (dict(delta=1.2), PARAM), (dict(klc=float("inf")), PARAM),
    (dict(enc=float("nan")), PARAM),
    (dict(ws=None), WORKSPACE), (dict(ws_bytes=4096), WORKSPACE),
])
def test_lmhead_aux_loss_rejects_bad_arguments_before_any_launch(over, expect):
    assert grpo.lib().grpo_lmhead_loss_aux_fwd_bwd(*lmhead_aux_args(**over)) == expect


def test_product_and_oracle_do_not_know_each_other():
    """The package imports nothing from oracle/ (and would have nothing to fall back on), the
    oracle imports nothing from the package, and the library's sources include no oracle file."""
    import ast
    import glob

    def imported(path):
        mods = set()
        for node in ast.walk(ast.parse(open(path).read())):
            if isinstance(node, ast.Import):
                mods.update(a.name.split(".")[0] for a in node.names)
            elif isinstance(node, ast.ImportFrom) and node.module and node.level == 0:
                mods.add(node.module.split(".")[0])
        return mods
    for f in glob.glob(os.path.join(ROOT, "paper_2505_07291_amd", "*.py")):
        assert "oracle" not in imported(f), f
    for f in glob.glob(os.path.join(ROOT, "oracle", "*.py")):
        assert "paper_2505_07291_amd" not in imported(f), f
    for f in glob.glob(os.path.join(ROOT, "paper_2505_07291_amd", "csrc", "*")) + \
            glob.glob(os.path.join(ROOT, "include", "*")):
        assert "oracle" not in open(f).read().lower(), f
    for f in glob.glob(os.path.join(ROOT, "oracle", "*.c")):
        includes = re.findall(r'#\s*include\s*[<"]([^>"]+)[>"]', open(f).read())
        assert includes and all("grpo" not in i and "hip" not in i for i in includes), (f, includes)
