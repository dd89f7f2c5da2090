"""GPU parity of the token-tree calls (psd_model_forward_tree, psd_tree_accept, psd_kv_compact_tree) against the CPU
oracle (oracle/forward.py forward_tree / compact_tree, oracle/tree.py) on the same seeded inputs.  Bars as for the
linear calls: bf16 logits rows within 2e-2 of the row's largest magnitude; paths and tokens bit-exact on every
sequence the near-tie flag does not excuse."""
import numpy as np
import pytest
import torch

from oracle import forward as ofwd
from oracle import tree as otree
from paper_2510_26527_amd import runtime, synth
import paper_2510_26527_amd as psd
from test_gpu_forward import Pair, check_logits, SMALL_GQA, SMALL_MHA

pytestmark = pytest.mark.gpu

TREES = {
    "chain5": [-1, 0, 1, 2, 3],
    "binary7": [-1, 0, 0, 1, 1, 2, 2],
    "wide_then_deep8": [-1, 0, 0, 0, 2, 4, 4, 5],
    "comb16": [-1] + [max(0, i - 2) for i in range(1, 16)],
    "full32": [-1] + [(i - 1) // 3 for i in range(1, 32)],
}


@pytest.mark.parametrize("shape,name,ctx,batch", [
    (SMALL_MHA, "chain5", 200, 1), (SMALL_MHA, "binary7", 1024, 1), (SMALL_MHA, "full32", 77, 2),
    (SMALL_GQA, "wide_then_deep8", 300, 3), (SMALL_GQA, "comb16", 129, 1), (SMALL_MHA, "comb16", 0, 1),
])
@pytest.mark.parametrize("pack", [False, True], ids=["rowmajor", "packed"])
def test_tree_forward_then_compaction_small_models(shape, name, ctx, batch, pack):
    """Every node's logits row, then the cache after keeping one accepted path per sequence: an ordinary step run on
    top of the compacted cache must match the oracle's (which was pinned to the pass over each root-to-node path)."""
    parents = TREES[name]
    n = len(parents)
    max_len = (ctx + n + 40 + 63) // 64 * 64
    lens = [max(ctx - 7 * b, 0) for b in range(batch)] if ctx else None
    p = Pair(shape, torch.bfloat16, batch, max_len, seed=n, ctx=ctx or None, lens=lens, std=0.05, pack=pack)
    toks = synth.make_tokens(shape.vocab, (batch, n + 5), n + ctx).astype(np.int32)
    base = p.kv.lens.clone()
    out = runtime.forward_tree(p.model, p.kv, torch.from_numpy(toks[:, :n]).cuda(), parents)
    torch.cuda.synchronize()
    obase = p.okv.lens.copy()
    ref = ofwd.forward_tree(p.cfg, p.w, toks[:, :n], parents, p.okv)
    e1 = check_logits(out, ref, torch.bfloat16, "tree rows")
    assert p.kv.lens.cpu().tolist() == (obase + n).tolist()
    # keep a root-to-leaf path in sequence 0, shorter ones (or nothing) in the others
    paths = []
    for b in range(batch):
        node, path = n - 1 - b, []
        while node > 0:
            path.append(node)
            node = parents[node]
        paths.append(path[::-1][:max(0, len(path) - b)])
    path_dev = torch.full((batch, n), -1, dtype=torch.int32)
    for b, path in enumerate(paths):
        path_dev[b, :len(path)] = torch.tensor(path, dtype=torch.int32)
    plen = torch.tensor([len(x) for x in paths], dtype=torch.int32)
    bound = int(max(int(obase[b]) + 1 + len(paths[b]) for b in range(batch)))
    psd.psd_kv_compact_tree(p.kv.handle, base, path_dev.cuda(), plen.cuda(), n, n, bound)
    ofwd.compact_tree(p.okv, obase, paths)
    torch.cuda.synchronize()
    assert p.kv.lens.cpu().tolist() == p.okv.lens.tolist()
    assert psd.psd_kv_len_upper_bound(p.kv.handle) == bound
    e2 = p.step(toks[:, n:], what="ordinary step on the compacted cache")
    print("rel err", e1, e2)
    p.close()


def test_tree_forward_limits():
    p = Pair(SMALL_GQA, torch.bfloat16, 1, 128, seed=3, ctx=20, std=0.05, pack=True)
    t = torch.zeros((1, 20), dtype=torch.int32, device="cuda")
    with pytest.raises(psd.PsdError):                      # a parent after its child
        runtime.forward_tree(p.model, p.kv, t[:, :4], [-1, 0, 3, 1])
    with pytest.raises(psd.PsdError):                      # no root
        runtime.forward_tree(p.model, p.kv, t[:, :3], [0, 0, 1])
    with pytest.raises(psd.PsdError):                      # group 2 x 20 nodes: more than the 32 query rows of the fused build
        runtime.forward_tree(p.model, p.kv, t, [-1] + list(range(19)))
    assert p.kv.lens.cpu().tolist() == [20]
    p.close()
    f = Pair(synth.TINY_TARGET, torch.float32, 1, 64, seed=1)
    with pytest.raises(psd.PsdError):                      # fp32 models have no fused attention build
        runtime.forward_tree(f.model, f.kv, t[:, :3], [-1, 0, 0])
    f.close()


def _accept_case(rows, name, V, dtype, seed, temperature, sharp=1.0):
    parents = TREES[name]
    n = len(parents)
    g = torch.Generator().manual_seed(seed)
    p = (torch.randn((rows, n, V), generator=g) * 2.0 * sharp).to(dtype)
    q = (p.float() + 0.7 * torch.randn((rows, n, V), generator=g)).to(dtype)
    # children's tokens: draws from the drafter's distribution at the parent (what the rule assumes), by Gumbel-max
    gum = -torch.log(-torch.log(torch.rand((rows, n, V), generator=g).clamp_min(1e-12)))
    toks = torch.zeros((rows, n), dtype=torch.int32)
    for i in range(1, n):
        toks[:, i] = torch.argmax(q[:, parents[i]].float() / max(temperature, 1e-3) + gum[:, i], dim=-1).to(torch.int32)
    u = torch.rand((rows, n + 1), generator=g)
    return parents, p, q, toks, u


@pytest.mark.parametrize("rows,name,V,dtype,temperature", [
    (8, "binary7", 1000, torch.float32, 1.0), (64, "wide_then_deep8", 32000, torch.bfloat16, 1.0),
    (5, "full32", 4099, torch.float32, 0.7), (16, "comb16", 32000, torch.float32, 1.3), (3, "chain5", 152064, torch.float32, 1.0),
    (33, "binary7", 517, torch.bfloat16, 1.0),
])
def test_tree_accept_matches_oracle(rows, name, V, dtype, temperature):
    parents, p, q, toks, u = _accept_case(rows, name, V, dtype, rows + V, temperature)
    out_len, out_path, out_tok, out_flags = runtime.tree_accept(p.cuda(), q.cuda(), toks.cuda(), parents, u.cuda(), temperature)
    torch.cuda.synchronize()
    out_len, out_path, out_tok, out_flags = [x.cpu().numpy() for x in (out_len, out_path, out_tok, out_flags)]
    pn, qn, un = p.float().numpy().astype(np.float64), q.float().numpy().astype(np.float64), u.numpy().astype(np.float64)
    excused, lens = 0, []
    for r in range(rows):
        path, tok, flags = otree.tree_accept(pn[r], qn[r], toks[r].numpy(), parents, un[r], temperature, return_flags=True)
        if flags & 1 or out_flags[r] & psd.PSD_FLAG_NEAR_TIE:
            excused += 1
            continue
        assert out_len[r] == len(path) and out_path[r, :len(path)].tolist() == path, (r, path, out_path[r])
        assert out_tok[r] == tok, (r, tok, out_tok[r])
        lens.append(len(path))
    assert excused <= max(1, rows // 16)
    print("accepted path lengths: mean %.2f, excused %d" % (np.mean(lens), excused))


def test_tree_accept_chain_is_the_linear_call():
    """One child per node: the same accepted length and token as psd_spec_accept on the same inputs."""
    rows, gamma, V = 32, 6, 32000
    parents = [-1] + list(range(gamma))
    g = torch.Generator().manual_seed(99)
    p = torch.randn((rows, gamma + 1, V), generator=g) * 2.0
    q = p + 0.5 * torch.randn((rows, gamma + 1, V), generator=g)
    toks = torch.zeros((rows, gamma + 1), dtype=torch.int32)
    gum = -torch.log(-torch.log(torch.rand((rows, gamma + 1, V), generator=g).clamp_min(1e-12)))
    for i in range(1, gamma + 1):
        toks[:, i] = torch.argmax(q[:, i - 1] + gum[:, i], dim=-1).to(torch.int32)
    u = torch.rand((rows, gamma + 2), generator=g)
    out_len, out_path, out_tok, _ = runtime.tree_accept(p.cuda(), q.cuda(), toks.cuda(), parents, u.cuda(), 1.0)
    acc = runtime.Acceptor("cuda")
    # the linear call: draft tokens x_1..x_gamma, proposal rows q_0..q_{gamma-1}, uniforms u_1..u_gamma then the draw's
    lin = acc(p.cuda(), q[:, :gamma].contiguous().cuda(), toks[:, 1:].contiguous().cuda(), u[:, 1:].contiguous().cuda(), 1.0)
    torch.cuda.synchronize()
    assert out_len.cpu().tolist() == lin[0].cpu().tolist()
    assert out_tok.cpu().tolist() == lin[1].cpu().tolist()
    for r in range(rows):
        assert out_path[r, :int(out_len[r])].cpu().tolist() == list(range(1, int(out_len[r]) + 1))


@pytest.mark.parametrize("rows,name,V,dtype", [(16, "full32", 32000, torch.bfloat16), (7, "wide_then_deep8", 1000, torch.float32)])
def test_tree_greedy_accept_matches_oracle(rows, name, V, dtype):
    parents, p, q, toks, u = _accept_case(rows, name, V, dtype, 5 * rows, 0.0, sharp=0.2)
    # plant the verifier's own choice on some children so that paths are not all empty
    top = torch.argmax(p.float(), dim=-1).to(torch.int32)
    for i in range(1, len(parents)):
        if i % 2:
            toks[:, i] = top[:, parents[i]]
    out_len, out_path, out_tok, _ = runtime.tree_accept(p.cuda(), None, toks.cuda(), parents, None, 0.0)
    torch.cuda.synchronize()
    pn = p.float().numpy().astype(np.float64)
    for r in range(rows):
        path, tok = otree.tree_greedy_accept(pn[r], toks[r].numpy(), parents)
        assert int(out_len[r]) == len(path) and out_path[r, :len(path)].cpu().tolist() == path
        assert int(out_tok[r]) == tok
    assert int(out_len.max()) >= 1


def test_whole_tree_step_on_a_small_model():
    """forward over the tree, acceptance on its logits, compaction, next step: the committed tokens and the next
    step's logits are those of the oracle doing the same."""
    shape, parents = SMALL_MHA, TREES["binary7"]
    n, batch = len(parents), 4
    p = Pair(shape, torch.bfloat16, batch, 256, seed=5, ctx=100, std=0.05, pack=True)
    toks = synth.make_tokens(shape.vocab, (batch, n), 3).astype(np.int32)
    base = p.kv.lens.clone()
    obase = p.okv.lens.copy()
    logits = runtime.forward_tree(p.model, p.kv, torch.from_numpy(toks).cuda(), parents)
    ref = ofwd.forward_tree(p.cfg, p.w, toks, parents, p.okv)
    check_logits(logits, ref, torch.bfloat16, "tree rows")
    g = torch.Generator().manual_seed(8)
    q = (logits.cpu() + 0.3 * torch.randn(logits.shape, generator=g)).cuda()      # a stand-in drafter close to the verifier
    u = torch.rand((batch, n + 1), generator=g)
    # both sides verify the GPU's own logits rows, as the chain tests do (1e-2 logit differences could flip a draw)
    out_len, out_path, out_tok, out_flags = runtime.tree_accept(logits, q, torch.from_numpy(toks).cuda(), parents, u.cuda(), 1.0)
    torch.cuda.synchronize()
    lg, qn = logits.cpu().double().numpy(), q.cpu().double().numpy()
    paths = []
    for b in range(batch):
        path, tok, flags = otree.tree_accept(lg[b], qn[b], toks[b], parents, u[b].double().numpy(), 1.0, return_flags=True)
        assert flags == 0 and int(out_flags[b]) == 0
        assert out_path[b, :int(out_len[b])].cpu().tolist() == path and int(out_tok[b]) == tok
        paths.append(path)
    bound = int(max(int(obase[b]) + 1 + len(paths[b]) for b in range(batch)))
    psd.psd_kv_compact_tree(p.kv.handle, base, out_path, out_len, n, n, bound)
    ofwd.compact_tree(p.okv, obase, paths)
    nxt = np.stack([np.concatenate([[int(out_tok[b])], synth.make_tokens(shape.vocab, (3,), 40 + b)]) for b in range(batch)])
    p.step(nxt.astype(np.int32), what="step after the tree")
    p.close()


def test_degenerate_trees():
    """A root alone (nothing drafted): the pass is an ordinary one-row step and the acceptance call is one draw from the
    verifier's row; a star (every node a child of the root): one level, up to 31 refusals against the running residual."""
    shape = SMALL_MHA
    p = Pair(shape, torch.bfloat16, 2, 128, seed=9, ctx=40, lens=[40, 17], std=0.05, pack=True)
    toks = synth.make_tokens(shape.vocab, (2, 1), 3).astype(np.int32)
    out = runtime.forward_tree(p.model, p.kv, torch.from_numpy(toks).cuda(), [-1])
    ref = ofwd.forward(p.cfg, p.w, toks, p.okv)
    check_logits(out, ref, torch.bfloat16, "root alone")
    u = torch.rand((2, 2), generator=torch.Generator().manual_seed(1))
    ln, path, tok, fl = runtime.tree_accept(out, out, torch.from_numpy(toks).cuda(), [-1], u.cuda(), 1.0)
    torch.cuda.synchronize()
    lg = out.cpu().double().numpy()
    for b in range(2):
        opath, otok = otree.tree_accept(lg[b], lg[b], toks[b], [-1], u[b].double().numpy(), 1.0)
        assert int(ln[b]) == 0 and opath == [] and int(tok[b]) == otok
    p.close()
    parents = [-1] + [0] * 31
    _, pl, ql, tk, uu = _accept_case(12, "full32", 2000, torch.float32, 77, 1.0)
    out_len, out_path, out_tok, out_flags = runtime.tree_accept(pl.cuda(), ql.cuda(), tk.cuda(), parents, uu.cuda(), 1.0)
    torch.cuda.synchronize()
    for r in range(12):
        path, tok, flags = otree.tree_accept(pl[r].double().numpy(), ql[r].double().numpy(), tk[r].numpy(), parents,
                                             uu[r].double().numpy(), 1.0, return_flags=True)
        if flags & 1 or int(out_flags[r]) & psd.PSD_FLAG_NEAR_TIE:
            continue
        assert out_path[r, :int(out_len[r])].cpu().tolist() == path and int(out_tok[r]) == tok


@pytest.mark.parametrize("name", ["binary7", "comb16"])
def test_tree_forward_on_a_4bit_model(name):
    """Two sequences: 14 rows in all (the streaming 4-bit projections) and 32 (the tiled ones)."""
    parents = TREES[name]
    n = len(parents)
    p = Pair(SMALL_GQA, torch.bfloat16, 2, 192, seed=4, ctx=100, std=0.05, w4=True)
    toks = synth.make_tokens(SMALL_GQA.vocab, (2, n), 5).astype(np.int32)
    out = runtime.forward_tree(p.model, p.kv, torch.from_numpy(toks).cuda(), parents)
    torch.cuda.synchronize()
    ref = ofwd.forward_tree(p.cfg, p.w, toks, parents, p.okv)
    print("rel err", check_logits(out, ref, torch.bfloat16, "4-bit tree rows"))
    p.close()


def test_tree_decoding_loop_small_models():
    """Several decoding steps with a drafted tree each: a drafter close to the verifier grows a binary tree of depth 2
    level by level (children = inverse-CDF draws from its own rows), the verifier runs one pass over the tree, the
    acceptance walks it, both caches keep the accepted path.  The oracle follows the verifier in lockstep: its rows
    after every compaction must match, and its acceptance on the same rows must commit the same tokens."""
    from oracle import accept as oacc
    shape, batch, steps = SMALL_MHA, 2, 6
    parents = [-1, 0, 0, 1, 1, 2, 2]
    n = len(parents)
    p = Pair(shape, torch.bfloat16, batch, 256, seed=31, ctx=60, lens=[60, 33], std=0.05, pack=True)
    g = torch.Generator().manual_seed(2)
    wd = {k: (v.float() + 0.03 * torch.randn(v.shape, generator=g)).to(v.dtype) if v.dtype == torch.bfloat16 and "norm" not in k else v
          for k, v in p.w.items()}
    draft = runtime.Model(shape, wd).pack()
    dkv = runtime.KVCache(draft, batch, 256)
    ks, vs = synth.make_kv_fill(shape, batch, 60, 32, torch.bfloat16)      # the drafter starts from the same context
    dkv.load(ks, vs, [60, 33])
    zero = torch.zeros(batch, dtype=torch.int32, device="cuda")
    root = synth.make_tokens(shape.vocab, (batch,), 4).astype(np.int32)
    tape = synth.make_uniforms((steps, batch, 6 + n + 1), 12).numpy().astype(np.float64)
    committed, longest = [[] for _ in range(batch)], 0
    for step in range(steps):
        base, dbase = p.kv.lens.clone(), dkv.lens.clone()
        obase = p.okv.lens.copy()
        toks = np.zeros((batch, n), np.int32)
        toks[:, 0] = root
        q = torch.zeros((batch, n, shape.vocab), dtype=torch.float32, device="cuda")
        # level 1: the drafter's row at the root, two independent draws from it
        q0 = runtime.forward_tree(draft, dkv, torch.from_numpy(toks[:, :1]).cuda(), [-1])
        psd.psd_kv_truncate(dkv.handle, dbase, zero, 0)
        q[:, 0] = q0[:, 0]
        for c in (1, 2):
            toks[:, c] = oacc.sample(q0[:, 0].cpu().numpy(), tape[step, :, c - 1])
        # level 2: its rows at the two children, two draws from each
        q12 = runtime.forward_tree(draft, dkv, torch.from_numpy(toks[:, :3]).cuda(), [-1, 0, 0])
        psd.psd_kv_truncate(dkv.handle, dbase, zero, 0)
        q[:, 1:3] = q12[:, 1:3]
        for c in (3, 4, 5, 6):
            toks[:, c] = oacc.sample(q12[:, parents[c]].cpu().numpy(), tape[step, :, c - 1])
        # the verifier's pass over the tree, checked against the oracle's on its own (compacted) cache
        t_dev = torch.from_numpy(toks).cuda()
        logits = runtime.forward_tree(p.model, p.kv, t_dev, parents)
        ref = ofwd.forward_tree(p.cfg, p.w, toks, parents, p.okv)
        check_logits(logits, ref, torch.bfloat16, f"step {step}")
        u = torch.from_numpy(tape[step, :, 6:].astype(np.float32))
        ln, path, tok, fl = runtime.tree_accept(logits, q, t_dev, parents, u.cuda(), 1.0)
        torch.cuda.synchronize()
        lg, qn = logits.cpu().double().numpy(), q.cpu().double().numpy()
        paths = []
        for b in range(batch):
            opath, otok, oflags = otree.tree_accept(lg[b], qn[b], toks[b], parents, u[b].double().numpy(), 1.0, return_flags=True)
            assert oflags == 0 and int(fl[b]) == 0
            assert path[b, :int(ln[b])].cpu().tolist() == opath and int(tok[b]) == otok, (step, b)
            committed[b] += [int(toks[b, c]) for c in opath] + [otok]
            paths.append(opath)
            longest = max(longest, len(opath))
        bound = int(max(int(obase[b]) + 1 + len(paths[b]) for b in range(batch)))
        psd.psd_kv_compact_tree(p.kv.handle, base, path, ln, n, n, bound)
        ofwd.compact_tree(p.okv, obase, paths)
        # the drafter re-reads the root and the accepted tokens (rows of different length: one sequence at a time would
        # be the plain way; here the longest path is fed and the lengths are cut back per sequence)
        width = 1 + max(len(x) for x in paths)
        feed = np.zeros((batch, width), np.int32)
        for b in range(batch):
            feed[b, :1 + len(paths[b])] = [toks[b, 0]] + [toks[b, c] for c in paths[b]]
        runtime.forward(draft, dkv, torch.from_numpy(feed).cuda(), 0)
        psd.psd_kv_truncate(dkv.handle, dbase, ln, 1)
        torch.cuda.synchronize()
        assert dkv.lens.cpu().tolist() == p.kv.lens.cpu().tolist() == p.okv.lens.tolist()
        root = tok.cpu().numpy().astype(np.int32)
    assert all(len(c) >= steps for c in committed) and longest >= 1, (committed, longest)
    print("tokens committed per sequence:", [len(c) for c in committed], "longest accepted path", longest)
    dkv.close()
    draft.close()
    p.close()
