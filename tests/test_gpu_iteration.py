"""One whole speculative-decoding iteration at temperature 0 (paper Section 2.1) on the GPU against
the same chain of CPU checker calls: the drafter decodes gamma tokens one at a time (embedding,
layers with one query position, vocabulary projection, arg-max draw), then the target scores the
last committed token plus the gamma drafts in one pass and the accept rule keeps a prefix.

Every arg-max of the chain is taken on logits that went through bf16 layers, so the comparison is
only meaningful where the checker's decision is clear: each case asserts that every arg-max of the
checker's chain leads the runner-up by GAP times the largest logit magnitude (ten times the error
the bf16 path shows on logits); the seeds below were chosen on the CPU to satisfy that."""
import numpy as np
import pytest
import torch

from oracle import verify_oracle as O
from paper_2505_10526_amd import synth, binding
from helpers import to_dev, i32, round_up, pad_rows
from test_gpu_layer import cfg_of

pytestmark = pytest.mark.gpu
GAP = 5e-3


class HostModel:
    """Weights and a prefilled cache of one synthetic model, as NumPy arrays."""

    def __init__(self, s, n_layers, B, kv_len, n_img, room, seed, w_std=0.05, head_std=0.05):
        self.s, self.n_layers = s, n_layers
        self.layers = [synth.layer_weights(s, seed, layer=l, std=w_std) for l in range(n_layers)]
        self.head = synth.lm_head_weights(s, seed, std=head_std)
        self.table = synth.embedding_table(s, seed)
        self.kv = [synth.kv_cache(s, B, room, kv_len, n_img, seed, layer=l, junk_tail=False) for l in range(n_layers)]
        self.kv_len = self.kv[0].kv_len.copy()
        self.n_img = self.kv[0].n_img.copy()


def oracle_forward(m, k, v, tokens, kv_len, pos):
    """tokens [B, Q] -> logits [B, Q, V]; k, v: lists of caches, updated in place."""
    B, Q = tokens.shape
    x = O.embed_tokens(m.table, tokens.reshape(-1)).reshape(B, Q, m.s.hidden)
    for l in range(m.n_layers):
        x, k[l], v[l] = O.verify_layer(m.s, m.layers[l], x, pos, k[l], v[l], kv_len)
    logits = O.lm_head_logits(x.reshape(B * Q, -1), m.head["final_norm"], m.head["w_lm"], m.s.norm_eps)
    return logits.reshape(B, Q, -1)


def clear_decisions(logits):
    top = np.sort(logits, axis=-1)[..., -2:]
    return np.all(top[..., 1] - top[..., 0] > GAP * np.max(np.abs(logits)))


def oracle_iteration(draft, target, last_tokens, gamma):
    B = len(last_tokens)
    kd = [kv.k.copy() for kv in draft.kv]; vd = [kv.v.copy() for kv in draft.kv]
    tok = np.asarray(last_tokens, dtype=np.int32)
    drafts = np.zeros((B, gamma), dtype=np.int32)
    clear = True
    for i in range(gamma):
        kv_len = draft.kv_len + i
        pos = synth.positions(kv_len, draft.n_img, 1, compress_image=True)
        logits = oracle_forward(draft, kd, vd, tok[:, None], kv_len, pos)
        clear &= clear_decisions(logits)
        _, out, _ = O.spec_accept(logits, None, np.zeros((B, 0), np.int32), None, 0.0)
        tok = out[:, 0].astype(np.int32)
        drafts[:, i] = tok
    kt = [kv.k.copy() for kv in target.kv]; vt = [kv.v.copy() for kv in target.kv]
    seq = np.concatenate([np.asarray(last_tokens, dtype=np.int32)[:, None], drafts], axis=1)
    pos = synth.positions(target.kv_len, target.n_img, gamma + 1, compress_image=True)
    logits = oracle_forward(target, kt, vt, seq, target.kv_len, pos)
    clear &= clear_decisions(logits)
    n, out, _ = O.spec_accept(logits, None, drafts, None, 0.0)
    return drafts, n, out, clear


class DeviceModel:
    def __init__(self, m):
        s = m.s
        self.m, self.cfg = m, cfg_of(s)
        self.l_max = round_up(m.kv[0].l_max, 32)
        self.k = [binding.k_cache_pack(to_dev(pad_rows(kv.k, self.l_max), s.dtype)) for kv in m.kv]
        self.v = [binding.v_cache_pack(to_dev(np.nan_to_num(pad_rows(kv.v, self.l_max)), s.dtype)) for kv in m.kv]
        ws = [binding.pack_layer_weights({k: (None if v is None else to_dev(v, s.dtype)) for k, v in w.items()})
              for w in m.layers]
        self.stack = binding.LayerStack(ws, self.k, self.v)
        self.norm = to_dev(m.head["final_norm"], s.dtype)
        self.w_lm = binding.weight_pack(to_dev(m.head["w_lm"], s.dtype))
        self.table = to_dev(m.table, s.dtype)

    def forward(self, tokens, kv_len, pos):
        B, Q = tokens.shape
        x = binding.embed_tokens(self.table, tokens.reshape(-1)).reshape(B, Q, -1)
        binding.verify_layers(self.cfg, self.stack, x, pos, kv_len, self.l_max)
        return binding.lm_head_logits(x, self.norm, self.w_lm, self.m.s.norm_eps).reshape(B, Q, -1)


def gpu_iteration(draft, target, last_tokens, gamma):
    B = len(last_tokens)
    d, t = DeviceModel(draft), DeviceModel(target)
    last = i32(last_tokens)
    tok = last.clone()
    drafts = torch.empty((B, gamma), dtype=torch.int32, device=last.device)
    for i in range(gamma):
        kv_len = draft.kv_len + i
        pos = synth.positions(kv_len, draft.n_img, 1, compress_image=True)
        logits = d.forward(tok.reshape(B, 1), i32(kv_len), i32(pos))
        _, out = binding.spec_accept(logits, None, None, None, 0.0)
        tok = out.reshape(B).clone()
        drafts[:, i] = tok
    seq = torch.cat([last.reshape(B, 1), drafts], dim=1).contiguous()
    pos = synth.positions(target.kv_len, target.n_img, gamma + 1, compress_image=True)
    logits = t.forward(seq, i32(target.kv_len), i32(pos))
    n, out = binding.spec_accept(logits, None, drafts.contiguous(), None, 0.0)
    torch.cuda.synchronize()
    return drafts.cpu().numpy(), n.cpu().numpy(), out.cpu().numpy()


def build_case(kind, seed, B=2, gamma=3):
    kv_len = [70, 33][:B]
    n_img = [40, 16][:B]
    target = HostModel(synth.TINY_BF16, 2, B, kv_len, n_img, gamma + 1, seed)
    if kind == "self":                       # the target drafts for itself: every draft is its own arg-max
        draft = target
    elif kind == "small":                    # an unrelated, smaller drafter: drafts are rarely accepted
        draft = HostModel(synth.TINY_DRAFT_BF16, 1, B, kv_len, n_img, gamma + 1, seed + 100)
    else:                                    # the target's layers under a perturbed vocabulary projection
        draft = HostModel(synth.TINY_BF16, 2, B, kv_len, n_img, gamma + 1, seed)
        noise = synth.normal(draft.head["w_lm"].shape, 0.015, seed, 77, dtype="bf16")
        draft.head = dict(draft.head, w_lm=synth.bf16_representable(draft.head["w_lm"] + noise))
    last = np.random.default_rng(seed).integers(0, target.s.vocab, B).astype(np.int32)
    return draft, target, last, gamma


CASES = [("self", 2), ("small", 0), ("noisy_head", 6), ("noisy_head", 17), ("noisy_head", 29)]


@pytest.mark.parametrize("kind,seed", CASES)
def test_greedy_iteration_matches_checker(kind, seed):
    draft, target, last, gamma = build_case(kind, seed)
    drafts_o, n_o, out_o, clear = oracle_iteration(draft, target, last, gamma)
    assert clear, "pick another seed: an arg-max of the checker's chain is too close to call"
    drafts_g, n_g, out_g = gpu_iteration(draft, target, last, gamma)
    assert np.array_equal(drafts_g, drafts_o)
    assert np.array_equal(n_g, n_o)
    assert np.array_equal(out_g, out_o)
    if kind == "self":
        assert np.all(n_o == gamma)


# ---------------------------------------------------------------------------
# several iterations in a row with the bookkeeping on the device (massv_commit_tokens)
# ---------------------------------------------------------------------------
def oracle_generation(draft, target, last_tokens, gamma, iterations):
    """Greedy decoding loop of Section 2.1.  Per iteration: gamma drafter steps, one more drafter forward on the
    last draft (so that the drafter's cache covers every token that can be kept), the target's verify pass, the
    accept rule, then kv_len += n + 1 and the final token becomes the next input."""
    B = len(last_tokens)
    kd = [kv.k.copy() for kv in draft.kv]; vd = [kv.v.copy() for kv in draft.kv]
    kt = [kv.k.copy() for kv in target.kv]; vt = [kv.v.copy() for kv in target.kv]
    kv_len = target.kv_len.copy()
    last = np.asarray(last_tokens, dtype=np.int32)
    emitted, clear = [[] for _ in range(B)], True
    for _ in range(iterations):
        tok, drafts = last.copy(), np.zeros((B, gamma), dtype=np.int32)
        for i in range(gamma + 1):
            pos = synth.positions(kv_len + i, draft.n_img, 1, compress_image=True)
            logits = oracle_forward(draft, kd, vd, tok[:, None], kv_len + i, pos)
            if i == gamma:
                break                                   # the extra forward only appends the last draft's cache row
            clear &= clear_decisions(logits)
            _, out, _ = O.spec_accept(logits, None, np.zeros((B, 0), np.int32), None, 0.0)
            tok = out[:, 0].astype(np.int32)
            drafts[:, i] = tok
        seq = np.concatenate([last[:, None], drafts], axis=1)
        pos = synth.positions(kv_len, target.n_img, gamma + 1, compress_image=True)
        logits = oracle_forward(target, kt, vt, seq, kv_len, pos)
        clear &= clear_decisions(logits)
        n, out, _ = O.spec_accept(logits, None, drafts, None, 0.0)
        for b in range(B):
            emitted[b].extend(out[b, : n[b] + 1].tolist())
        last, kv_len = O.commit_tokens(n, out, kv_len)
    return emitted, kv_len, clear


def gpu_generation(draft, target, last_tokens, gamma, iterations):
    B = len(last_tokens)
    d, t = DeviceModel(draft), DeviceModel(target)
    kv_len = i32(target.kv_len)
    img_half = i32(target.n_img // 2)                   # rotary ids count the image prefix as half its length
    last = i32(last_tokens)
    steps = torch.arange(gamma + 1, dtype=torch.int32, device=last.device)
    records = []
    for _ in range(iterations):
        tok = last.clone()
        drafts = torch.empty((B, gamma), dtype=torch.int32, device=last.device)
        for i in range(gamma + 1):
            kv_i = (kv_len + i).contiguous()
            pos_i = (kv_i - img_half).reshape(B, 1).contiguous()
            logits = d.forward(tok.reshape(B, 1), kv_i, pos_i)
            if i == gamma:
                break
            _, out = binding.spec_accept(logits, None, None, None, 0.0)
            tok = out.reshape(B).clone()
            drafts[:, i] = tok
        seq = torch.cat([last.reshape(B, 1), drafts], dim=1).contiguous()
        pos = ((kv_len - img_half).reshape(B, 1) + steps.reshape(1, -1)).contiguous()
        logits = t.forward(seq, kv_len, pos)
        n, out = binding.spec_accept(logits, None, drafts.contiguous(), None, 0.0)
        records.append((n.clone(), out.clone()))
        last = binding.commit_tokens(n, out, kv_len)    # kv_len advances in place, no host round trip
    torch.cuda.synchronize()
    emitted = [[] for _ in range(B)]
    for n, out in records:
        n, out = n.cpu().numpy(), out.cpu().numpy()
        for b in range(B):
            emitted[b].extend(out[b, : n[b] + 1].tolist())
    return emitted, kv_len.cpu().numpy()


def build_generation_case(seed, iterations=3, gamma=3, B=2):
    kv_len, n_img = [70, 33][:B], [40, 16][:B]
    room = iterations * (gamma + 1) + 1
    target = HostModel(synth.TINY_BF16, 2, B, kv_len, n_img, room, seed)
    draft = HostModel(synth.TINY_BF16, 2, B, kv_len, n_img, room, seed)
    noise = synth.normal(draft.head["w_lm"].shape, 0.015, seed, 77, dtype="bf16")
    draft.head = dict(draft.head, w_lm=synth.bf16_representable(draft.head["w_lm"] + noise))
    last = np.random.default_rng(seed).integers(0, target.s.vocab, B).astype(np.int32)
    return draft, target, last, gamma, iterations


@pytest.mark.parametrize("seed", [4, 34])
def test_greedy_generation_over_three_iterations(seed):
    draft, target, last, gamma, iterations = build_generation_case(seed)
    em_o, kv_o, clear = oracle_generation(draft, target, last, gamma, iterations)
    assert clear, "pick another seed: an arg-max of the checker's chain is too close to call"
    em_g, kv_g = gpu_generation(draft, target, last, gamma, iterations)
    assert em_g == em_o
    assert np.array_equal(kv_g, kv_o)
    assert any(len(e) > iterations for e in em_o)       # some drafts were accepted along the way
