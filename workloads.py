"""Seeded synthetic workloads (inputs only; none of the method's arithmetic).

The five configurations stand in for the paper's model pairs and prompts
(Llama-3, Qwen-2.5, Gemma-3 logits on its benchmark prompts, Sec. 4.1), none of
which are available here: vocabulary sizes are those model families' public
sizes, tree shapes are root expansion (Sec. 3.2) and delayed expansion (Sec. 5,
Def. 5.2), temperatures come from the paper's sampling grid.  Logit rows are
independent draws per (tree, node); draft tokens are drawn i.i.d. from the
softmax of the parent's stored draft row at the run's temperature, which is the
drafting assumption of Sec. 3.2.

Everything is generated with torch on the requested device from fixed seeds and
handed, unchanged, both to the library and (copied to the host) to the oracle.
"""

from dataclasses import dataclass, field
from typing import List

import torch

from paper_2602_16994_amd.trees import delayed_tree

SPECINFER = 0
TRAVERSAL = 1
NSS = 2
NAIVE = 3
SPECTR = 4


@dataclass
class Config:
    name: str
    B: int
    V: int
    K: int
    L1: int
    L2: int
    dtype: str            # "f32" | "bf16"
    T: float
    methods: List[int]
    draft_sigma: float
    target_sigma: float
    target_scale: float = 1.0
    gumbel_scale: float = 0.0      # z_d = gumbel_scale*Gumbel + N(0, draft_sigma^2)
    top_boost_k: int = 0           # add top_boost to the row's top_boost_k largest entries
    top_boost: float = 0.0
    seed: int = 0
    parent: List[int] = field(default_factory=list)

    def __post_init__(self):
        self.parent = delayed_tree(self.K, self.L1, self.L2)

    @property
    def N(self):
        return len(self.parent)

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def elem_bytes(self):
        return 4 if self.dtype == "f32" else 2


CONFIGS = {
    # 1: tiny, root expansion k=2 depth 3 (7 nodes)
    "tiny": Config("tiny", B=1, V=1024, K=2, L1=0, L2=3, dtype="f32", T=1.0,
                   methods=[SPECINFER, TRAVERSAL], draft_sigma=2.0, target_sigma=0.5, seed=1007),
    # 2: B=64, V=32000, root expansion k=4 depth 4 (17 nodes), heavy head
    "v32k_root": Config("v32k_root", B=64, V=32000, K=4, L1=0, L2=4, dtype="f32", T=1.0,
                        methods=[SPECINFER], draft_sigma=1.0, target_sigma=0.8, gumbel_scale=3.0,
                        top_boost_k=50, top_boost=4.0, seed=2007),
    # 3: B=64, V=128256, delayed: trunk 2, then k=4 branches of depth 3 (15 nodes)
    "v128k_delayed": Config("v128k_delayed", B=64, V=128256, K=4, L1=2, L2=3, dtype="bf16", T=0.6,
                            methods=[SPECINFER, TRAVERSAL], draft_sigma=1.0, target_sigma=1.0,
                            gumbel_scale=3.0, top_boost_k=50, top_boost=4.0, seed=3007),
    # 4: B=256, V=151936, root expansion k=8 depth 5 (41 nodes)  -- the benchmark line
    "v152k_root": Config("v152k_root", B=256, V=151936, K=8, L1=0, L2=5, dtype="bf16", T=1.0,
                         methods=[TRAVERSAL], draft_sigma=2.5, target_sigma=1.2,
                         top_boost_k=20, top_boost=5.0, seed=4007),
    # 5: B=32, V=262144, delayed: trunk 3, then k=8 branches of depth 3 (28 nodes)
    "v262k_delayed": Config("v262k_delayed", B=32, V=262144, K=8, L1=3, L2=3, dtype="bf16", T=0.8,
                            methods=[SPECINFER, TRAVERSAL], draft_sigma=3.0, target_sigma=1.5,
                            target_scale=0.8, seed=5007),
}


def scaled(cfg, **over):
    """A copy of cfg with some fields replaced (e.g. a smaller B or V for tests)."""
    d = {k: getattr(cfg, k) for k in (
        "name", "B", "V", "K", "L1", "L2", "dtype", "T", "methods", "draft_sigma", "target_sigma",
        "target_scale", "gumbel_scale", "top_boost_k", "top_boost", "seed")}
    d.update(over)
    return Config(**d)


def _rows(cfg, rows, gen, device):
    """rows x V draft and target logits in float32, before rounding to the stored dtype."""
    V = cfg.V
    zd = torch.randn(rows, V, generator=gen, device=device) * cfg.draft_sigma
    if cfg.gumbel_scale:
        u = torch.rand(rows, V, generator=gen, device=device).clamp_(1e-20, 1.0)
        zd += cfg.gumbel_scale * (-torch.log((-torch.log(u)).clamp_(min=1e-20)))
    if cfg.top_boost_k:
        idx = torch.topk(zd, min(cfg.top_boost_k, V), dim=1).indices
        zd.scatter_add_(1, idx, torch.full(idx.shape, cfg.top_boost, device=device))
    zt = cfg.target_scale * zd + torch.randn(rows, V, generator=gen, device=device) * cfg.target_sigma
    return zd, zt


def make_inputs(cfg, device="cuda", trees_per_chunk=8):
    """Returns dict(parent, tokens[B,N] int32, target[B,N,V], draft[B,N,V], uniforms[B,N] f32,
    draw_uniforms[B,N] f32 (the second set, for the methods that draw a token at every node)).

    Logits are generated chunk by chunk in float32 and stored in cfg's dtype.
    """
    B, N, V = cfg.B, cfg.N, cfg.V
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(cfg.seed)
    target = torch.empty(B, N, V, dtype=cfg.torch_dtype, device=dev)
    draft = torch.empty(B, N, V, dtype=cfg.torch_dtype, device=dev)
    for b0 in range(0, B, trees_per_chunk):
        b1 = min(B, b0 + trees_per_chunk)
        zd, zt = _rows(cfg, (b1 - b0) * N, gen, dev)
        draft[b0:b1] = zd.view(b1 - b0, N, V).to(cfg.torch_dtype)
        target[b0:b1] = zt.view(b1 - b0, N, V).to(cfg.torch_dtype)
        del zd, zt

    # draft tokens: i.i.d. from softmax(stored draft row of the parent / T)
    gen_tok = torch.Generator(device=dev)
    gen_tok.manual_seed(cfg.seed + 1)
    tokens = torch.zeros(B, N, dtype=torch.int32, device=dev)
    for n in range(1, N):
        par = cfg.parent[n]
        for b0 in range(0, B, 64):
            b1 = min(B, b0 + 64)
            q = torch.softmax(draft[b0:b1, par].float() / cfg.T, dim=-1)
            tokens[b0:b1, n] = torch.multinomial(q, 1, generator=gen_tok).squeeze(1).to(torch.int32)

    gen_u = torch.Generator(device=dev)
    gen_u.manual_seed(cfg.seed + 2)
    uniforms = torch.rand(B, N, generator=gen_u, device=dev, dtype=torch.float32)
    gen_d = torch.Generator(device=dev)
    gen_d.manual_seed(cfg.seed + 3)
    draw_uniforms = torch.rand(B, N, generator=gen_d, device=dev, dtype=torch.float32)
    return {"parent": list(cfg.parent), "tokens": tokens, "target": target, "draft": draft,
            "uniforms": uniforms, "draw_uniforms": draw_uniforms}


def make_context_inputs(cfg, device="cuda"):
    """make_inputs for models that are functions of the context (Sec. 3, Def. 3.1): slots of one
    tree that were drafted for the same context (same tokens from the root down) hold the same
    target row and the same draft row, and draft tokens are drawn from the row of the context.
    Logit rows and uniforms are those of make_inputs(cfg); walking the slots in ascending order,
    the token of slot n is drawn from the (already final) draft row of its parent slot, and if an
    earlier slot of the tree has the same context, that slot's two rows are copied into slot n.
    Adds "context_node" (numpy int32 [B,N]): the first slot drafted for slot n's context.
    """
    import numpy as np
    inputs = make_inputs(cfg, device)
    B, N = cfg.B, cfg.N
    dev = torch.device(device)
    target, draft = inputs["target"], inputs["draft"]
    gen_tok = torch.Generator(device=dev)
    gen_tok.manual_seed(cfg.seed + 1)
    tokens = torch.zeros(B, N, dtype=torch.int32, device=dev)
    first_slot = [dict() for _ in range(B)]           # per tree: (context's slot, token) -> first slot drafted for it
    context_node = np.zeros((B, N), dtype=np.int32)
    for n in range(1, N):
        par = cfg.parent[n]
        for b0 in range(0, B, 64):
            b1 = min(B, b0 + 64)
            q = torch.softmax(draft[b0:b1, par].float() / cfg.T, dim=-1)
            tokens[b0:b1, n] = torch.multinomial(q, 1, generator=gen_tok).squeeze(1).to(torch.int32)
        drawn = tokens[:, n].cpu().tolist()
        again_b, again_m = [], []
        for b in range(B):
            m = first_slot[b].setdefault((int(context_node[b, par]), drawn[b]), n)
            context_node[b, n] = m
            if m != n:
                again_b.append(b)
                again_m.append(m)
        if again_b:
            ib = torch.tensor(again_b, device=dev)
            im = torch.tensor(again_m, device=dev)
            draft[ib, n] = draft[ib, im]
            target[ib, n] = target[ib, im]
    inputs["tokens"] = tokens
    inputs["context_node"] = context_node
    return inputs


def reorder_trees(inputs, order):
    """The same batch with its trees in another order (order: a permutation of range(B))."""
    idx = torch.as_tensor(list(order), device=inputs["tokens"].device, dtype=torch.long)
    out = dict(inputs)
    for k in ("tokens", "target", "draft", "uniforms", "draw_uniforms"):
        out[k] = inputs[k].index_select(0, idx).contiguous()
    if "context_node" in inputs:
        out["context_node"] = inputs["context_node"][list(order)]
    return out


def to_host(inputs):
    """numpy copies for the oracle (bfloat16 widened to float32, which is exact)."""
    host = {
        "parent": inputs["parent"],
        "tokens": inputs["tokens"].cpu().numpy(),
        "target": inputs["target"].float().cpu().numpy(),
        "draft": inputs["draft"].float().cpu().numpy(),
        "uniforms": inputs["uniforms"].cpu().numpy(),
    }
    if "draw_uniforms" in inputs:
        host["draw_uniforms"] = inputs["draw_uniforms"].cpu().numpy()
    return host
