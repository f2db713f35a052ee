"""Seeded synthetic model-shaped tensor sets (inputs only, no method arithmetic).

Stands in for the paper's trained checkpoints (its evaluation lists OPT,
LLaMA, Qwen, Yi and GPT models from 1.3B to 20B parameters, Section 5.1):
what the Load path consumes is parameter bytes, so each model here is a list
of named bf16 tensors with the shapes of its family, filled from a seeded
generator.  Both the HIP path and the CPU oracle read the bytes produced
here; this module computes no fingerprint, plan or copy.

Values: fp32 N(0, 0.02) rounded to bf16 (round to nearest even), or the bf16
constant 1.0 for normalisation gains where a workload asks for it.  A tensor's
bytes are a function of its ``content`` seed, its element count and the
device the generator runs on ("cpu" and "cuda" give different streams; within
one run one device is used throughout).  Two tensors with equal content seed
and shape are byte-identical: that is how sibling models share tensors.
"""
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import torch

BF16_BYTES = 2


@dataclass(frozen=True)
class TensorSpec:
    name: str
    shape: Tuple[int, ...]
    kind: str          # "normal" or "ones"
    content: int       # generator seed; ignored for "ones"

    @property
    def numel(self) -> int:
        n = 1
        for d in self.shape:
            n *= d
        return n

    @property
    def nbytes(self) -> int:
        return self.numel * BF16_BYTES


@dataclass
class ModelSpec:
    name: str
    model_id: int
    tensors: List[TensorSpec]

    @property
    def nbytes(self) -> int:
        return sum(t.nbytes for t in self.tensors)


@dataclass
class Workload:
    """A pool, the models that touch it, and the order of operations.

    ``setup`` runs once; ``loads`` are the measured loads.  An action is
    ("load", model_name) or ("release", model_name, evict).  After each
    measured load the loader releases the model with eviction so the pool is
    back in its post-setup state.
    """
    name: str
    pool_bytes: int
    align: int
    models: Dict[str, ModelSpec]
    setup: List[tuple]
    loads: List[str]
    designated_shared: Dict[str, int] = field(default_factory=dict)
    # True when models larger than the pinned Model Cache are registered without
    # a host image and reach the pool segment by segment
    streamed: bool = False
    # plan flags for the measured loads: any of "evict", "merge", "alias"
    load_flags: Dict[str, bool] = field(default_factory=dict)
    # True when a measured load changes the pool beyond what releasing the model
    # undoes (it moved or evicted residents): the setup is replayed before each step
    rebuild_each_step: bool = False
    # eviction-cost parameters (miss probability, load bandwidth, sensitivity) by model name
    costs: Dict[str, Tuple[float, float, float]] = field(default_factory=dict)


def seed_for(cfg: int, model: int, k: int) -> int:
    return 1000003 * (1000 * cfg + model) + k


# --------------------------------------------------------------- tensor lists
def gpt_tensors(h: int, layers: int, ffn: int, vocab: int, positions: int
                ) -> List[Tuple[str, Tuple[int, ...], bool]]:
    """GPT-2/OPT-style list; (name, shape, is_norm_gain).  Output head tied."""
    out = [("tok_embed", (vocab, h), False), ("pos_embed", (positions, h), False)]
    for i in range(layers):
        p = "l%d." % i
        out += [
            (p + "ln1.g", (h,), True), (p + "ln1.b", (h,), False),
            (p + "qkv.w", (3 * h, h), False), (p + "qkv.b", (3 * h,), False),
            (p + "out.w", (h, h), False), (p + "out.b", (h,), False),
            (p + "ln2.g", (h,), True), (p + "ln2.b", (h,), False),
            (p + "up.w", (ffn, h), False), (p + "up.b", (ffn,), False),
            (p + "down.w", (h, ffn), False), (p + "down.b", (h,), False),
        ]
    out += [("lnf.g", (h,), True), ("lnf.b", (h,), False)]
    return out


def llama_tensors(h: int, layers: int, ffn: int, vocab: int, kv_dim: int
                  ) -> List[Tuple[str, Tuple[int, ...], bool]]:
    """Llama-style list with RMSNorm gains and an untied lm_head."""
    out = [("embed", (vocab, h), False)]
    for i in range(layers):
        p = "l%d." % i
        out += [
            (p + "in_norm", (h,), True),
            (p + "q", (h, h), False), (p + "k", (kv_dim, h), False),
            (p + "v", (kv_dim, h), False), (p + "o", (h, h), False),
            (p + "post_norm", (h,), True),
            (p + "gate", (ffn, h), False), (p + "up", (ffn, h), False),
            (p + "down", (h, ffn), False),
        ]
    out += [("final_norm", (h,), True), ("lm_head", (vocab, h), False)]
    return out


def neox_tensors(h: int, layers: int, ffn: int, vocab: int
                 ) -> List[Tuple[str, Tuple[int, ...], bool]]:
    """GPT-NeoX-style list (rotary positions, untied embed_out)."""
    out = [("embed_in", (vocab, h), False)]
    for i in range(layers):
        p = "l%d." % i
        out += [
            (p + "ln1.g", (h,), True), (p + "ln1.b", (h,), False),
            (p + "ln2.g", (h,), True), (p + "ln2.b", (h,), False),
            (p + "qkv.w", (3 * h, h), False), (p + "qkv.b", (3 * h,), False),
            (p + "dense.w", (h, h), False), (p + "dense.b", (h,), False),
            (p + "h4h.w", (ffn, h), False), (p + "h4h.b", (ffn,), False),
            (p + "4hh.w", (h, ffn), False), (p + "4hh.b", (h,), False),
        ]
    out += [("lnf.g", (h,), True), ("lnf.b", (h,), False),
            ("embed_out", (vocab, h), False)]
    return out


def layer_of(name: str) -> Optional[int]:
    if name.startswith("l") and "." in name and name[1:name.index(".")].isdigit():
        return int(name[1:name.index(".")])
    return None


def make_model(name: str, model_id: int, shapes, cfg: int, model_no: int,
               gains_one: bool, share_from: Optional[ModelSpec] = None,
               shared=lambda k, nm: False, subset=None) -> ModelSpec:
    """Build a ModelSpec.  Tensor k takes its content seed from
    ``share_from`` when ``shared(k, name)`` holds, else a seed of its own.
    ``subset(k, name)`` keeps only part of the list (a partially resident
    model)."""
    tensors = []
    for k, (nm, shape, is_gain) in enumerate(shapes):
        if subset is not None and not subset(k, nm):
            continue
        if is_gain and gains_one:
            tensors.append(TensorSpec(nm, shape, "ones", 0))
        elif share_from is not None and shared(k, nm):
            src = next(t for t in share_from.tensors if t.name == nm)
            tensors.append(TensorSpec(nm, shape, src.kind, src.content))
        else:
            tensors.append(TensorSpec(nm, shape, "normal",
                                      seed_for(cfg, model_no, k)))
    return ModelSpec(name, model_id, tensors)


# ------------------------------------------------------------------ workloads
GIB = 1 << 30
MIB = 1 << 20


def workload_tiny() -> Workload:
    """Config 1: tiny GPT-shaped pair, 75 % of tensors byte-identical."""
    shapes = gpt_tensors(256, 4, 1024, 4096, 1024)
    a = make_model("A", 1, shapes, 1, 0, gains_one=False)
    b = make_model("B", 2, shapes, 1, 1, gains_one=False, share_from=a,
                   shared=lambda k, nm: k % 4 != 3)
    return Workload("tiny-gpt-pair", 64 * MIB, 256, {"A": a, "B": b},
                    [("load", "A"), ("release", "A", False)], ["B"],
                    {"B": sum(1 for k in range(len(shapes)) if k % 4 != 3)})


def workload_gpt1b() -> Workload:
    """Config 2: 1.3B GPT-shaped model; a sibling shares embeddings and the
    even layers."""
    shapes = gpt_tensors(2048, 24, 8192, 50304, 2048)
    s = make_model("S", 1, shapes, 2, 0, gains_one=True)

    def shared(k, nm):
        lay = layer_of(nm)
        return nm in ("tok_embed", "pos_embed") or (lay is not None and lay % 2 == 0)
    m = make_model("M", 2, shapes, 2, 1, gains_one=True, share_from=s,
                   shared=shared)
    n_shared = sum(1 for k, (nm, _, _) in enumerate(shapes) if shared(k, nm))
    return Workload("gpt-1.3b-sibling", 8 * GIB, 256, {"S": s, "M": m},
                    [("load", "S"), ("release", "S", False)], ["M"],
                    {"M": n_shared})


def workload_llama7b() -> Workload:
    """Config 3: 7B Llama-shaped base and three variants sharing embeddings,
    lm_head and layers 0-15."""
    shapes = llama_tensors(4096, 32, 11008, 32000, 4096)
    base = make_model("base", 1, shapes, 3, 0, gains_one=True)

    def shared(k, nm):
        lay = layer_of(nm)
        return nm in ("embed", "lm_head") or (lay is not None and lay < 16)
    models = {"base": base}
    for v in (1, 2, 3):
        models["v%d" % v] = make_model("v%d" % v, 1 + v, shapes, 3, v,
                                       gains_one=True, share_from=base,
                                       shared=shared)
    n_shared = sum(1 for k, (nm, _, _) in enumerate(shapes) if shared(k, nm))
    return Workload("llama-7b-family", 64 * GIB, 256, models,
                    [("load", "base"), ("release", "base", False)],
                    ["v1", "v2", "v3"], {"v%d" % v: n_shared for v in (1, 2, 3)})


def workload_neox20b() -> Workload:
    """Config 4: 20B NeoX-shaped model into a 200 GB pool that holds five
    resident models with holes between them; 30 % of its tensors match a
    resident partial sibling."""
    shapes20 = neox_tensors(6144, 44, 24576, 50432)
    residents = [
        ("R1", gpt_tensors(2048, 24, 8192, 50304, 2048)),
        ("R2", gpt_tensors(2560, 32, 10240, 50304, 2048)),
        ("R3", gpt_tensors(4096, 32, 16384, 50304, 2048)),
        ("R4", gpt_tensors(5120, 40, 20480, 50304, 2048)),
    ]
    models: Dict[str, ModelSpec] = {}
    setup: List[tuple] = []
    # fillers of different depths leave holes of different sizes once evicted
    filler_layers = [6, 10, 14, 18, 24]
    mid = 1

    def in_r5(k, nm):
        lay = layer_of(nm)
        return nm in ("embed_in", "lnf.g", "lnf.b") or (lay is not None and lay <= 12)
    r5 = make_model("R5", 5, shapes20, 4, 5, gains_one=True, subset=in_r5)
    for i, (nm, shp) in enumerate(residents):
        models[nm] = make_model(nm, mid, shp, 4, i + 1, gains_one=True)
        mid += 1
    models["R5"] = r5
    for i, fl in enumerate(filler_layers):
        fn = "F%d" % (i + 1)
        models[fn] = make_model(fn, 50 + i, gpt_tensors(2048, fl, 8192, 50304, 2048),
                                4, 20 + i, gains_one=True)
    order = ["R1", "F1", "R2", "F2", "R3", "F3", "R4", "F4", "R5", "F5"]
    for nm in order:
        setup.append(("load", nm))
        setup.append(("release", nm, False))
    for i in range(len(filler_layers)):
        setup.append(("release", "F%d" % (i + 1), True))
    m20 = make_model("M20", 100, shapes20, 4, 9, gains_one=True, share_from=r5,
                     shared=lambda k, nm: in_r5(k, nm))
    models["M20"] = m20
    n_shared = sum(1 for k, (nm, _, _) in enumerate(shapes20) if in_r5(k, nm))
    return Workload("neox-20b-fragmented", 200 * 10**9 // 256 * 256, 256, models,
                    setup, ["M20"], {"M20": n_shared})


def workload_neox20b_tight(pool_gb: float = 72.0) -> Workload:
    """Config 4's models in a pool that is too small: the five residents
    (59.4 GB, all retained, none running) leave 12.6 GB free and the 20B model
    needs 28.7 GB of new slots in alias mode.  Stage 1 has to evict by cost,
    Stage 2 has to merge what eviction leaves fragmented.  Cost parameters per
    resident are in `costs` (miss probability, bandwidth, sensitivity)."""
    base = workload_neox20b()
    models = {k: v for k, v in base.models.items() if not k.startswith("F")}
    setup: List[tuple] = []
    for nm in ("R1", "R2", "R3", "R4", "R5"):
        setup += [("load", nm), ("release", nm, False)]
    w = Workload("neox-20b-tight-pool", int(pool_gb * 1e9) // 256 * 256, 256, models, setup, ["M20"],
                 dict(base.designated_shared))
    w.load_flags = {"evict": True, "merge": True, "alias": True, "pack_text": True}
    w.rebuild_each_step = True
    w.costs = {"R1": (1.0, 57e9, 1.0), "R2": (0.8, 57e9, 1.0), "R3": (0.2, 57e9, 1.0),
               "R4": (0.5, 57e9, 1.0), "R5": (1.0, 57e9, 1.0)}
    return w


def _llama70b_keep(reuse: float):
    """Which tensors a 70B model shares with its resident sibling at a designated reuse level."""
    if reuse <= 0.0:
        return lambda k, nm: False
    if reuse <= 0.5:
        def keep50(k, nm):
            lay = layer_of(nm)
            return nm == "embed" or (lay is not None and lay < 40)
        return keep50

    def keep90(k, nm):
        lay = layer_of(nm)
        return nm in ("embed", "lm_head", "final_norm") or (lay is not None and lay < 72)
    return keep90


LLAMA70B_SHAPES = dict(h=8192, layers=80, ffn=28672, vocab=128256, kv_dim=1024)


def workload_llama70b(reuse: float, pool_bytes: int) -> Workload:
    """Config 5: 70B Llama-3-shaped model (723 tensors, 141 GB) loaded as one
    model; a resident sibling holds the designated share of its tensors (0, 50
    or 90 %).  Neither fits pinned host memory at once, so both are registered
    without a host image and pass through the Model Cache segment by segment
    (`streamed`)."""
    shapes = llama_tensors(**LLAMA70B_SHAPES)
    keep = _llama70b_keep(reuse)
    models: Dict[str, ModelSpec] = {}
    setup: List[tuple] = []
    sib = make_model("sib", 1, shapes, 5, 0, gains_one=True, subset=keep)
    if sib.tensors:
        models["sib"] = sib
        setup += [("load", "sib"), ("release", "sib", False)]
    models["M70"] = make_model("M70", 2, shapes, 5, 1, gains_one=True,
                               share_from=sib if sib.tensors else None, shared=keep)
    n_shared = sum(1 for k, (nm, _, _) in enumerate(shapes) if keep(k, nm))
    w = Workload("llama3-70b-reuse%02d" % int(round(reuse * 100)),
                 pool_bytes // 256 * 256, 256, models, setup, ["M70"], {"M70": n_shared})
    w.streamed = True
    return w


def workload_llama70b_sweep(pool_bytes: int, levels=(0.9, 0.5, 0.0)) -> Workload:
    """Config 5's three reuse levels against one pool: the resident sibling is
    the 90 % one (embeddings, lm_head, final norm, layers 0-71: 127 GB); the
    model measured at level r shares with it exactly the tensors designated for
    r and brings its own bytes for the rest.  Loads are named "M70-<percent>"."""
    shapes = llama_tensors(**LLAMA70B_SHAPES)
    sib = make_model("sib", 1, shapes, 5, 0, gains_one=True, subset=_llama70b_keep(0.9))
    models: Dict[str, ModelSpec] = {"sib": sib}
    loads, shared = [], {}
    for i, r in enumerate(levels):
        keep = _llama70b_keep(r)
        name = "M70-%d" % int(round(r * 100))
        models[name] = make_model(name, 2 + i, shapes, 5, 1, gains_one=True, share_from=sib, shared=keep)
        loads.append(name)
        shared[name] = sum(1 for k, (nm, _, _) in enumerate(shapes) if keep(k, nm))
    w = Workload("llama3-70b-sweep", pool_bytes // 256 * 256, 256, models,
                 [("load", "sib"), ("release", "sib", False)], loads, shared)
    w.streamed = True
    return w


def workload_merge(hole_mib: int = 320, residents: int = 16, resident_mib: int = 1024,
                   new_tensors: int = 4, new_mib: int = 1000, tail_mib: int = 3072,
                   pack_text: bool = True) -> Workload:
    """`residents` retained tensors of resident_mib MiB, each followed by a hole
    of hole_mib MiB, then a free tail of tail_mib MiB.  The incoming model's
    tensors (new_mib MiB each) fit the free bytes but not all of them fit the
    tail and none fits a hole, so best fit fails and Stage 2 has to merge free
    regions by moving residents."""
    mib = 1 << 20
    models: Dict[str, ModelSpec] = {}
    setup: List[tuple] = []
    for i in range(residents):
        k = ModelSpec("K%d" % i, 10 + i, [TensorSpec("k%d" % i, (resident_mib * mib // 2,), "normal",
                                                     seed_for(6, i, 0))])
        h = ModelSpec("H%d" % i, 500 + i, [TensorSpec("h%d" % i, (hole_mib * mib // 2,), "normal",
                                                      seed_for(6, 100 + i, 0))])
        models[k.name], models[h.name] = k, h
        setup += [("load", k.name), ("release", k.name, False), ("load", h.name), ("release", h.name, False)]
    for i in range(residents):
        setup.append(("release", "H%d" % i, True))
    n = ModelSpec("N", 1000, [TensorSpec("n%d" % j, (new_mib * mib // 2 - 8 * j,), "normal", seed_for(6, 200, j))
                              for j in range(new_tensors)])
    models["N"] = n
    pool = (residents * (resident_mib + hole_mib) + tail_mib) * mib
    w = Workload("merge-holes-%dMiB" % hole_mib, pool, 256, models, setup, ["N"])
    w.load_flags = {"merge": True, "pack_text": pack_text}
    w.rebuild_each_step = True
    return w


WORKLOADS = {
    "tiny": workload_tiny,
    "gpt1b": workload_gpt1b,
    "llama7b": workload_llama7b,
    "neox20b": workload_neox20b,
    "neox20b-tight": workload_neox20b_tight,
    "merge": workload_merge,
    "merge-listing": lambda: workload_merge(pack_text=False),
    "merge-notail": lambda: workload_merge(tail_mib=0),
    "merge-small": lambda: workload_merge(hole_mib=16, residents=16, resident_mib=512, new_tensors=2,
                                          new_mib=120, tail_mib=0),
}


# ------------------------------------------------------------------ generator
_ONE_BF16 = 0x3F80


def tensor_bytes(spec: TensorSpec, device: str = "cpu") -> torch.Tensor:
    """The tensor's bytes as a 1-D uint8 tensor on ``device``."""
    if spec.kind == "ones":
        t = torch.full((spec.numel,), 1.0, dtype=torch.bfloat16, device=device)
    elif spec.kind == "normal":
        g = torch.Generator(device=device)
        g.manual_seed(spec.content)
        t = torch.randn(spec.numel, generator=g, device=device,
                        dtype=torch.float32)
        t = t.mul_(0.02).to(torch.bfloat16)
    else:
        raise ValueError(spec.kind)
    return t.view(torch.uint8)


def layout(model: ModelSpec, align: int = 256) -> List[int]:
    """Offsets of the model's tensors in its host (Model Cache) buffer, packed
    in list order with each tensor starting on an ``align`` boundary."""
    offs = []
    at = 0
    for t in model.tensors:
        offs.append(at)
        at += (t.nbytes + align - 1) // align * align
    return offs


def host_bytes(model: ModelSpec, align: int = 256) -> int:
    offs = layout(model, align)
    if not offs:
        return 0
    last = model.tensors[-1].nbytes
    return offs[-1] + (last + align - 1) // align * align


def fill_host(model: ModelSpec, out: torch.Tensor, device: str = "cpu",
              align: int = 256) -> List[int]:
    """Write every tensor of ``model`` into ``out`` (a 1-D uint8 CPU tensor of
    at least ``host_bytes(model)`` bytes, usually pinned) and return the
    offsets.  Generation runs on ``device``."""
    offs = layout(model, align)
    for t, off in zip(model.tensors, offs):
        out[off:off + t.nbytes].copy_(tensor_bytes(t, device))
    return offs


def shared_layout(models: Sequence[ModelSpec], align: int = 256):
    """One Model Cache image for several models in which tensors with equal
    content (see content_key) are stored once.  Returns (total bytes,
    {model name: [offset per tensor]}, [(TensorSpec, offset)] of the unique
    tensors in first-seen order)."""
    at = 0
    seen = {}
    per_model = {}
    unique = []
    for m in models:
        offs = []
        for t in m.tensors:
            key = content_key(t)
            if key not in seen:
                seen[key] = at
                unique.append((t, at))
                at += (t.nbytes + align - 1) // align * align
            offs.append(seen[key])
        per_model[m.name] = offs
    return max(at, align), per_model, unique


def content_key(spec: TensorSpec) -> Tuple:
    """Identity of a tensor's bytes: equal keys <=> equal bytes (for a given
    device).  Lets metadata-only tests stand in a fake fingerprint."""
    if spec.kind == "ones":
        return ("ones", spec.numel)
    return ("normal", spec.content, spec.numel)
