"""Per-architecture tensor tables: the model description the estimator consumes.

The paper obtains, for a pre-trained decoder, (i) its parameter tensors classed
Embedding / Linear / Bias / LayerNorm and split into input embedding, lm_head and
"the rest" (Notation table; Sec. 4.2, text after the m_p and m_os equations) and
(ii) the output size of every operator as a function of batch size and sequence
length (Sec. 3.1, computation-graph extraction).  Here both are *data*: a list of
`ParamEntry` and a list of `EventEntry` per architecture family.  Every size is a
monomial  coef * prod(D[dim])  over the per-configuration dimension vector D
(`DIMS` below); nothing in this module evaluates one.

The event list is the fine-tuning iteration of Sec. 4.1 / 4.2 under gradient
checkpointing, written as signed allocator events in five segments:

  A  once   embedding outputs (kept for the whole iteration)
  F  x L    forward of one transformer block, intermediates freed, output kept
  H  once   final norm, lm_head logits, the two shifted copies, loss, loss backward
  B  x L    backward of one block: recompute, gradients, all-gather buffers (TP),
            then the block's kept output is freed
  Z  once   release of what A/H/B left alive, optimizer temporaries

With `checkpoint=False` the builders give the iteration without gradient
checkpointing, the full traversal of the computation graph that Sec. 3.1
describes for DNNMem: F allocates every operator output of a block and keeps
what autograd saves (and the block output) alive, B is the backward alone, and
nothing is recomputed, so live ranges span the whole forward pass.

The per-family operator lists are synthetic stand-ins of the shape a graph
extraction of GPT-2 / OPT / LLaMA style blocks yields (about 60 operators per
block counting forward and recompute); they are inputs, not part of the method.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

# ---------------------------------------------------------------------------
# vocabulary shared by every consumer of a table (pure naming, no arithmetic)
# ---------------------------------------------------------------------------
DIMS: Tuple[str, ...] = (
    "one", "bs", "sl", "sl_m1", "h", "ffn", "n_heads", "n_kv",
    "head_dim", "kv_dim", "V", "P", "L", "B_logits", "d",
)
DIM_INDEX: Dict[str, int] = {n: i for i, n in enumerate(DIMS)}

CLASSES = ("E", "L", "B", "N")          # Embedding, Linear, Bias, LayerNorm/RMSNorm
ROLES = ("EMBED_TOK", "LM_HEAD", "OTHER")
SEGMENTS = ("A", "F", "H", "B", "Z")
METHODS = ("CDP", "ZERO3", "TP")        # ids 0, 1, 2
ALL_METHODS = frozenset((0, 1, 2))
SCALES = ("none", "tp_gather")          # tp_gather: raw -> ceil(raw * (d-1) / d)


@dataclass(frozen=True)
class ParamEntry:
    name: str
    coef: int
    dims: Tuple[str, ...]               # at most 4 names from DIMS
    cls: str                            # one of CLASSES
    role: str                           # one of ROLES
    per_layer: bool                     # True: one such tensor in each of the L blocks


@dataclass(frozen=True)
class EventEntry:
    name: str
    seg: str                            # one of SEGMENTS
    sign: int                           # +1 allocation, -1 release
    coef: int
    dims: Tuple[str, ...]
    elem_bytes: int
    methods: frozenset = ALL_METHODS    # event exists only under these methods
    scale: str = "none"
    times_L: bool = False               # L equal blocks handled by one event


@dataclass(frozen=True)
class ArchTable:
    name: str
    params: Tuple[ParamEntry, ...]
    events: Tuple[EventEntry, ...]


# ---------------------------------------------------------------------------
# operator lists -> event lists (bookkeeping of lifetimes only)
# ---------------------------------------------------------------------------
@dataclass
class Op:
    """One operator output: `size` = (coef, dims, elem_bytes); `last` names the
    operator after which the tensor is dead in a no-grad forward; `saved` marks
    tensors autograd keeps for the backward when the block is recomputed;
    `wgrad` gives the size of a transient weight-gradient tensor the backward of
    this operator materialises (Linear operators)."""
    name: str
    size: Tuple[int, Tuple[str, ...], int]
    last: str
    saved: bool = False
    wgrad: Tuple[int, Tuple[str, ...], int] | None = None


def _ev(name, seg, sign, size, **kw) -> EventEntry:
    coef, dims, eb = size
    return EventEntry(name, seg, sign, coef, tuple(dims), eb, **kw)


def _forward_events(ops: Sequence[Op], seg: str, keep: str) -> List[EventEntry]:
    """No-grad forward: allocate each output, free a tensor right after its last
    consumer has produced its own output; `keep` (the block output) survives."""
    names = [o.name for o in ops]
    assert len(set(names)) == len(names)
    out: List[EventEntry] = []
    for i, o in enumerate(ops):
        out.append(_ev(o.name, seg, +1, o.size))
        for p in ops[: i + 1]:
            if p.last == o.name and p.name != keep:
                out.append(_ev("free:" + p.name, seg, -1, p.size))
    freed = {e.name[5:] for e in out if e.sign < 0}
    for p in ops:
        assert p.name == keep or p.name in freed, f"{p.name} never freed"
    return out


def _backward_events(ops: Sequence[Op], seg: str, x_size, tp_size) -> List[EventEntry]:
    """Backward of one recomputed block.

    Recompute: the forward again, but tensors autograd saved stay alive.  Then the
    operators in reverse: materialise the gradient w.r.t. the operator's output
    consumer (same size as the output), a transient weight gradient for Linear
    operators, the backward all-gather buffer of 1-D tensor parallelism (Sec. 5,
    m_back^tp: kept until the backward has finished, so it is *not* freed here),
    then drop the previous gradient and the saved activation.  Last, the block's
    kept output (its checkpoint) is released.
    """
    out: List[EventEntry] = _saving_forward_events(ops, seg, "re:")
    return out + _gradient_events(ops, seg, x_size, tp_size, free_checkpoint=True)


def _saving_forward_events(ops: Sequence[Op], seg: str, prefix: str) -> List[EventEntry]:
    """Forward of one block with autograd recording: every output is allocated, a
    tensor is freed after its last consumer unless autograd saved it."""
    out: List[EventEntry] = []
    for i, o in enumerate(ops):
        out.append(_ev(prefix + o.name, seg, +1, o.size))
        for p in ops[: i + 1]:
            if p.last == o.name and not p.saved:
                out.append(_ev("free:" + prefix + p.name, seg, -1, p.size))
    return out


def _gradient_events(ops: Sequence[Op], seg: str, x_size, tp_size, free_checkpoint: bool) -> List[EventEntry]:
    """The operators of one block in reverse (see `_backward_events`); what the
    forward with autograd left alive is released on the way; with
    `free_checkpoint` the block's separately kept output goes last."""
    out: List[EventEntry] = []
    alive = [p for p in ops if p.saved or p.last not in {q.name for q in ops}]
    alive_names = {p.name for p in alive}
    # the incoming gradient dY (size of the block output) was allocated before
    prev = ("dY", x_size)
    for o in reversed(ops):
        out.append(_ev("grad:" + o.name, seg, +1, o.size))
        if o.wgrad is not None:
            out.append(_ev("wgrad:" + o.name, seg, +1, o.wgrad))
            out.append(_ev("free:wgrad:" + o.name, seg, -1, o.wgrad))
        out.append(_ev("free:" + prev[0], seg, -1, prev[1]))
        prev = ("grad:" + o.name, o.size)
        if o.name in alive_names:
            out.append(_ev("free:saved:" + o.name, seg, -1, o.size))
    # the last gradient produced is the dY handed to the block below: rename only
    assert prev[1] == x_size, "first operator of a block must have the block-input size"
    out.append(_ev("tp_allgather_buf", seg, +1, tp_size,
                   methods=frozenset((2,)), scale="tp_gather"))
    if free_checkpoint:
        out.append(_ev("free:kept_block_output", seg, -1, x_size))
    return out


# ---------------------------------------------------------------------------
# size shorthands (coef, dims, elem_bytes)
# ---------------------------------------------------------------------------
def _X(eb=2):      return (1, ("bs", "sl", "h"), eb)
def _TOK(eb=4):    return (1, ("bs", "sl"), eb)
def _KV(eb=2):     return (1, ("bs", "sl", "kv_dim"), eb)
def _S(eb=2):      return (1, ("bs", "n_heads", "sl", "sl"), eb)
def _FF(eb=2):     return (1, ("bs", "sl", "ffn"), eb)
def _ROPE(eb=2):   return (1, ("sl", "head_dim"), eb)
def _W(a, b, eb=2): return (1, (a, b), eb)


def _attention_ops(fused_kv_dim: str, rope: bool) -> List[Op]:
    """Self-attention operators shared by the families (eager attention)."""
    ops = [
        Op("q_proj", _X(), "q_heads", wgrad=_W("h", "h")),
        Op("k_proj", (1, ("bs", "sl", fused_kv_dim), 2), "k_heads", wgrad=_W("h", fused_kv_dim)),
        Op("v_proj", (1, ("bs", "sl", fused_kv_dim), 2), "v_heads", wgrad=_W("h", fused_kv_dim)),
        Op("q_heads", _X(), "q_rot" if rope else "scores", saved=not rope),
        Op("k_heads", (1, ("bs", "sl", fused_kv_dim), 2), "k_rot" if rope else "k_rep"),
        Op("v_heads", (1, ("bs", "sl", fused_kv_dim), 2), "v_rep"),
    ]
    if rope:
        ops += [
            Op("rope_cos", _ROPE(), "k_rot"),
            Op("rope_sin", _ROPE(), "k_rot"),
            Op("q_half", _X(), "q_rot"),
            Op("q_rot", _X(), "scores", saved=True),
            Op("k_half", (1, ("bs", "sl", fused_kv_dim), 2), "k_rot"),
            Op("k_rot", (1, ("bs", "sl", fused_kv_dim), 2), "k_rep"),
        ]
    ops += [
        Op("k_rep", _X(), "scores", saved=True),
        Op("v_rep", _X(), "attn_ctx", saved=True),
        Op("scores", _S(), "scores_scaled"),
        Op("scores_scaled", _S(), "scores_masked"),
        Op("scores_masked", _S(), "softmax_f32"),
        Op("softmax_f32", _S(4), "probs"),
        Op("probs", _S(), "probs_drop", saved=True),
        Op("probs_drop", _S(), "attn_ctx", saved=True),
        Op("attn_ctx", _X(), "attn_merge"),
        Op("attn_merge", _X(), "o_proj", saved=True),
        Op("o_proj", _X(), "resid1", wgrad=_W("h", "h")),
    ]
    return ops


def _layernorm_ops(tag: str, nxt: str) -> List[Op]:
    return [
        Op(f"{tag}_f32", _X(4), f"{tag}_norm"),
        Op(f"{tag}_mean", _TOK(), f"{tag}_norm", saved=True),
        Op(f"{tag}_cent", _X(4), f"{tag}_norm"),
        Op(f"{tag}_rstd", _TOK(), f"{tag}_norm", saved=True),
        Op(f"{tag}_norm", _X(4), f"{tag}_out"),
        Op(f"{tag}_out", _X(), nxt, saved=True),
    ]


def _rmsnorm_ops(tag: str, nxt: str) -> List[Op]:
    return [
        Op(f"{tag}_f32", _X(4), f"{tag}_norm", saved=True),
        Op(f"{tag}_sq", _X(4), f"{tag}_var"),
        Op(f"{tag}_var", _TOK(), f"{tag}_norm", saved=True),
        Op(f"{tag}_norm", _X(4), f"{tag}_cast"),
        Op(f"{tag}_cast", _X(), f"{tag}_out", saved=True),
        Op(f"{tag}_out", _X(), nxt, saved=True),
    ]


def _gpt_block(act: str) -> List[Op]:
    ops = _layernorm_ops("ln1", "v_proj")
    ops += _attention_ops("h", rope=False)
    ops += [Op("resid1", _X(), "resid2", saved=False)]
    ops += _layernorm_ops("ln2", "fc1")
    ops += [Op("fc1", _FF(), "act_out", saved=True, wgrad=_W("h", "ffn"))]
    if act == "gelu":
        ops += [
            Op("gelu_cube", _FF(), "gelu_inner"),
            Op("gelu_inner", _FF(), "gelu_tanh"),
            Op("gelu_tanh", _FF(), "act_out", saved=True),
        ]
    ops += [
        Op("act_out", _FF(), "fc2", saved=True),
        Op("fc2", _X(), "fc2_drop", wgrad=_W("ffn", "h")),
        Op("fc2_drop", _X(), "resid2", saved=True),
        Op("resid2", _X(), "<block output>"),
    ]
    return ops


def _llama_block() -> List[Op]:
    ops = _rmsnorm_ops("ln1", "v_proj")
    ops += _attention_ops("kv_dim", rope=True)
    ops += [Op("resid1", _X(), "resid2")]
    ops += _rmsnorm_ops("ln2", "up_proj")
    ops += [
        Op("gate_proj", _FF(), "gate_act", saved=True, wgrad=_W("h", "ffn")),
        Op("gate_act", _FF(), "glu_mul", saved=True),
        Op("up_proj", _FF(), "glu_mul", saved=True, wgrad=_W("h", "ffn")),
        Op("glu_mul", _FF(), "down_proj", saved=True),
        Op("down_proj", _X(), "resid2", wgrad=_W("ffn", "h")),
        Op("resid2", _X(), "<block output>"),
    ]
    return ops


def _fix_first(ops: List[Op]) -> List[Op]:
    """The first operator's output must have block-input size so the gradient
    chain of the backward ends in a dY of that size (it does: an fp32 copy of x is
    not; so prepend the identity view the block receives)."""
    return [Op("block_in_view", _X(), ops[0].name)] + ops


def _head_events(norm: str) -> List[EventEntry]:
    """Final norm, lm_head and loss (Sec. 4.2, m_lm): logits, the two shifted
    copies (shifted logits, and their log-softmax), loss backward."""
    LOG = (1, ("bs", "sl", "V", "B_logits"), 1)
    SH = (1, ("bs", "sl_m1", "V", "B_logits"), 1)
    LAB = (1, ("bs", "sl_m1"), 8)
    ev: List[EventEntry] = []
    norm_ops = _layernorm_ops("lnf", "lm_logits") if norm == "layernorm" else _rmsnorm_ops("lnf", "lm_logits")
    for e in _forward_events(norm_ops + [Op("lm_logits", LOG, "<kept>")], "H", "lm_logits"):
        ev.append(e)
    ev += [
        _ev("shift_logits", "H", +1, SH),
        _ev("shift_labels", "H", +1, LAB),
        _ev("log_softmax", "H", +1, SH),
        _ev("nll_per_token", "H", +1, (1, ("bs", "sl_m1"), 4)),
        _ev("loss", "H", +1, (1, ("one",), 4)),
        _ev("free:nll_per_token", "H", -1, (1, ("bs", "sl_m1"), 4)),
        # loss backward: gradient of log-softmax reuses the shifted-logit buffer
        _ev("free:log_softmax", "H", -1, SH),
        _ev("grad_logits", "H", +1, LOG),
        _ev("free:shift_logits", "H", -1, SH),
        _ev("free:shift_labels", "H", -1, LAB),
        _ev("free:lm_logits", "H", -1, LOG),
        _ev("dY_final", "H", +1, _X()),
        _ev("wgrad:lm_head", "H", +1, _W("V", "h")),
        _ev("free:wgrad:lm_head", "H", -1, _W("V", "h")),
        _ev("free:grad_logits", "H", -1, LOG),
        _ev("free:loss", "H", -1, (1, ("one",), 4)),
    ]
    return ev


def _tail_events(n_embed: int, opt_tmp) -> List[EventEntry]:
    ev = [_ev("free:dY", "Z", -1, _X())]
    for i in range(n_embed):
        ev.append(_ev(f"free:embed_out{i}", "Z", -1, _X()))
    ev.append(_ev("free:tp_allgather_bufs", "Z", -1, _X(), methods=frozenset((2,)),
                  scale="tp_gather", times_L=True))
    # optimizer step: an fp32 working copy of the largest tensor, twice (update, then cast)
    ev += [
        _ev("adam_tmp_update", "Z", +1, opt_tmp),
        _ev("adam_tmp_denom", "Z", +1, opt_tmp),
        _ev("free:adam_tmp_denom", "Z", -1, opt_tmp),
        _ev("free:adam_tmp_update", "Z", -1, opt_tmp),
    ]
    return ev


def _assemble(name: str, params: List[ParamEntry], n_embed: int, block: List[Op], norm: str,
              checkpoint: bool = True) -> ArchTable:
    block = _fix_first(block)
    ev: List[EventEntry] = []
    for i in range(n_embed):
        ev.append(_ev(f"embed_out{i}", "A", +1, _X()))
    if n_embed > 1:
        ev.append(_ev("embed_sum", "A", +1, _X()))
        ev.append(_ev("free:embed_sum", "A", -1, _X()))
    if checkpoint:
        ev += _forward_events(block, "F", block[-1].name)
        ev += _head_events(norm)
        ev += _backward_events(block, "B", _X(), _X())
    else:
        ev += _saving_forward_events(block, "F", "")
        ev += _head_events(norm)
        ev += _gradient_events(block, "B", _X(), _X(), free_checkpoint=False)
    ev += _tail_events(n_embed, (1, ("V", "h"), 4))
    return ArchTable(name, tuple(params), tuple(ev))


def _gpt_params() -> List[ParamEntry]:
    P = ParamEntry
    p = [
        P("wte", 1, ("V", "h"), "E", "EMBED_TOK", False),
        P("wpe", 1, ("P", "h"), "E", "OTHER", False),
    ]
    for nm in ("q", "k", "v", "o"):
        p.append(P(f"attn.{nm}.weight", 1, ("h", "h"), "L", "OTHER", True))
        p.append(P(f"attn.{nm}.bias", 1, ("h",), "B", "OTHER", True))
    p += [
        P("mlp.fc1.weight", 1, ("h", "ffn"), "L", "OTHER", True),
        P("mlp.fc1.bias", 1, ("ffn",), "B", "OTHER", True),
        P("mlp.fc2.weight", 1, ("ffn", "h"), "L", "OTHER", True),
        P("mlp.fc2.bias", 1, ("h",), "B", "OTHER", True),
        P("ln1.weight", 1, ("h",), "N", "OTHER", True),
        P("ln1.bias", 1, ("h",), "N", "OTHER", True),
        P("ln2.weight", 1, ("h",), "N", "OTHER", True),
        P("ln2.bias", 1, ("h",), "N", "OTHER", True),
        P("ln_f.weight", 1, ("h",), "N", "OTHER", False),
        P("ln_f.bias", 1, ("h",), "N", "OTHER", False),
        P("lm_head.weight", 1, ("V", "h"), "L", "LM_HEAD", False),
    ]
    return p


def _llama_params() -> List[ParamEntry]:
    P = ParamEntry
    return [
        P("embed_tokens", 1, ("V", "h"), "E", "EMBED_TOK", False),
        P("q_proj", 1, ("h", "h"), "L", "OTHER", True),
        P("k_proj", 1, ("h", "kv_dim"), "L", "OTHER", True),
        P("v_proj", 1, ("h", "kv_dim"), "L", "OTHER", True),
        P("o_proj", 1, ("h", "h"), "L", "OTHER", True),
        P("gate_proj", 1, ("h", "ffn"), "L", "OTHER", True),
        P("up_proj", 1, ("h", "ffn"), "L", "OTHER", True),
        P("down_proj", 1, ("ffn", "h"), "L", "OTHER", True),
        P("input_layernorm", 1, ("h",), "N", "OTHER", True),
        P("post_attention_layernorm", 1, ("h",), "N", "OTHER", True),
        P("norm", 1, ("h",), "N", "OTHER", False),
        P("lm_head", 1, ("V", "h"), "L", "LM_HEAD", False),
    ]


def gpt_table(checkpoint: bool = True) -> ArchTable:
    """GPT-2 style: learned positions, biases, LayerNorm, tanh-GELU MLP."""
    return _assemble("gpt" if checkpoint else "gpt_full", _gpt_params(), 2, _gpt_block("gelu"), "layernorm", checkpoint)


def opt_table(checkpoint: bool = True) -> ArchTable:
    """OPT style: as GPT but a ReLU MLP."""
    return _assemble("opt" if checkpoint else "opt_full", _gpt_params(), 2, _gpt_block("relu"), "layernorm", checkpoint)


def llama_table(checkpoint: bool = True) -> ArchTable:
    """LLaMA style: RMSNorm, rotary embedding, grouped-query attention, SwiGLU, no biases."""
    return _assemble("llama" if checkpoint else "llama_full", _llama_params(), 1, _llama_block(), "rmsnorm", checkpoint)


def degenerate_table(base: ArchTable) -> ArchTable:
    """Same parameters, but a timeline holding only what the paper's closed form
    counts and releasing nothing: embedding outputs, one kept output per block,
    logits and the two shifted copies (Sec. 4.2, m_out and m_lm)."""
    n_embed = sum(1 for p in base.params if p.cls == "E" and p.role != "LM_HEAD")
    ev = [_ev(f"embed_out{i}", "A", +1, _X()) for i in range(n_embed)]
    ev.append(_ev("block_out", "F", +1, _X()))
    ev.append(_ev("lm_logits", "H", +1, (1, ("bs", "sl", "V", "B_logits"), 1)))
    ev.append(_ev("shift_logits", "H", +1, (1, ("bs", "sl_m1", "V", "B_logits"), 1)))
    ev.append(_ev("log_softmax", "H", +1, (1, ("bs", "sl_m1", "V", "B_logits"), 1)))
    return ArchTable(base.name + "_degenerate", base.params, tuple(ev))


def random_table(rng, n_param: int, n_event: int, name: str = "random", n_sizes: int = 0) -> ArchTable:
    """A structurally valid but arbitrary table (for parity tests): random
    selectors, classes, roles, signs, method masks, scales and segment lengths.
    With n_sizes > 0 the events draw their size expression (coefficient,
    dimensions, element width, method mask, scaling) from a pool of that many.
    `rng` is a numpy Generator."""
    large = ("sl", "sl_m1", "h", "ffn", "P", "kv_dim")          # at most two of these per size: no int64 overflow
    tiny = ("one", "bs", "n_heads", "n_kv", "head_dim", "L", "B_logits", "d")
    params = []
    for i in range(n_param):
        nd = int(rng.integers(0, 3))
        dims = tuple(str(rng.choice(("h", "ffn", "V", "P", "kv_dim", "head_dim", "n_heads", "one"))) for _ in range(nd))
        params.append(ParamEntry(f"p{i}", int(rng.integers(1, 5)), dims,
                                 str(rng.choice(CLASSES)), str(rng.choice(ROLES)), bool(rng.integers(0, 2))))

    def size_spec():
        dims = tuple(str(rng.choice(large)) for _ in range(int(rng.integers(0, 3)))) \
            + tuple(str(rng.choice(tiny)) for _ in range(int(rng.integers(0, 3))))
        mask = frozenset(m for m in (0, 1, 2) if rng.integers(0, 4) > 0)
        return (int(rng.integers(1, 9)), dims, int(rng.choice((1, 2, 4, 8))), mask,
                "tp_gather" if rng.integers(0, 6) == 0 else "none", bool(rng.integers(0, 8) == 0))

    pool = [size_spec() for _ in range(n_sizes)]
    cuts = sorted(int(x) for x in rng.integers(0, n_event + 1, size=4))
    bounds = [0] + cuts + [n_event]
    events = []
    for s, seg in enumerate(SEGMENTS):
        for i in range(bounds[s], bounds[s + 1]):
            coef, dims, eb, mask, scale, times_l = pool[int(rng.integers(0, n_sizes))] if n_sizes else size_spec()
            if n_sizes:
                dims = tuple(rng.permutation(list(dims))) if dims else dims    # same product, other order
            events.append(EventEntry(f"e{i}", seg, +1 if rng.integers(0, 5) > 1 else -1, coef,
                                     tuple(str(x) for x in dims), eb, mask, scale, times_l))
    return ArchTable(name, tuple(params), tuple(events))


FAMILIES = {"gpt": gpt_table, "opt": opt_table, "llama": llama_table}


@dataclass(frozen=True)
class Constants:
    """Constants of the estimator that are inputs, not fixed by the method
    (Notation table: m_base, cu_p; Sec. 3.1: the 512-byte block of the allocator)."""
    m_base: int = 0
    cu_p: int = 2 * 1024 * 1024
    align: int = 512
