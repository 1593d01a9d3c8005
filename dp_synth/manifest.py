"""Layer manifests (shapes only) of the workloads: one dense layer, BERT-Base- and
BERT-Large-shaped stacks.  A manifest is an ordered list of LayerSpec; the flat
parameter space is the concatenation, in manifest order, of each layer's tensors in
the order given by LayerSpec.tensors()."""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple


@dataclass(frozen=True)
class LayerSpec:
    name: str
    kind: str  # "dense" | "layernorm" | "embedding" | "tied_embedding"
    d_in: int = 0  # dense: input width; embedding: number of rows V
    d_out: int = 0  # dense: output width; layernorm/embedding: width d
    has_bias: bool = False
    distinct: bool = False  # embedding: ids are distinct within an example (position ids)
    segment: bool = False  # embedding: token-type ids (0 for the first half of the sequence, 1 for the second)
    grad_group: str = ""  # layers with the same non-empty group receive ONE output-gradient tensor (the three
                          # embedding tables are summed before their LayerNorm, so they share its input gradient)
    n_pred: int = 0  # tied_embedding: prediction slots M per example whose logits use the table as output projection

    def tensors(self) -> List[Tuple[str, Tuple[int, ...]]]:
        if self.kind == "dense":
            t = [(self.name + ".W", (self.d_in, self.d_out))]
            if self.has_bias:
                t.append((self.name + ".b", (self.d_out,)))
            return t
        if self.kind == "layernorm":
            return [(self.name + ".gamma", (self.d_out,)), (self.name + ".beta", (self.d_out,))]
        if self.kind in ("embedding", "tied_embedding"):
            return [(self.name + ".E", (self.d_in, self.d_out))]
        raise ValueError(self.kind)

    def param_count(self) -> int:
        n = 0
        for _, shp in self.tensors():
            k = 1
            for s in shp:
                k *= s
            n += k
        return n


def single_dense_manifest(d_in: int, d_out: int, has_bias: bool = False) -> List[LayerSpec]:
    return [LayerSpec("dense0", "dense", d_in, d_out, has_bias)]


def bert_manifest(n_layers: int, hidden: int, ffn: int, vocab: int = 0, max_pos: int = 0, tied_pred: int = 0,
                  type_vocab: int = 0) -> List[LayerSpec]:
    """Per block: Q, K, V, O dense hidden x hidden, LayerNorm, FFN hidden x ffn and ffn x hidden,
    LayerNorm; all dense layers carry biases. Optional token and position embeddings first.  With tied_pred = M
    the token table is also the output projection of M prediction slots per example (one parameter, two uses).
    With type_vocab = 2 the embedding stage is the full one of Section 4.3: word-piece, positional and token-type
    tables whose lookups are summed (one shared output gradient) and the LayerNorm that follows the sum."""
    m: List[LayerSpec] = []
    grp = "emb" if type_vocab else ""
    if vocab and tied_pred:
        m.append(LayerSpec("emb.tok", "tied_embedding", vocab, hidden, n_pred=tied_pred, grad_group=grp))
    elif vocab:
        m.append(LayerSpec("emb.tok", "embedding", vocab, hidden, grad_group=grp))
    if max_pos:
        m.append(LayerSpec("emb.pos", "embedding", max_pos, hidden, distinct=True, grad_group=grp))
    if type_vocab:
        m.append(LayerSpec("emb.type", "embedding", type_vocab, hidden, segment=True, grad_group=grp))
        m.append(LayerSpec("emb.ln", "layernorm", 0, hidden))
    for l in range(n_layers):
        p = f"block{l}."
        for nm in ("q", "k", "v", "o"):
            m.append(LayerSpec(p + nm, "dense", hidden, hidden, True))
        m.append(LayerSpec(p + "ln1", "layernorm", 0, hidden))
        m.append(LayerSpec(p + "ffn1", "dense", hidden, ffn, True))
        m.append(LayerSpec(p + "ffn2", "dense", ffn, hidden, True))
        m.append(LayerSpec(p + "ln2", "layernorm", 0, hidden))
    return m


def manifest_param_count(m: List[LayerSpec]) -> int:
    return sum(l.param_count() for l in m)


# The five workloads. "dtype" is the type of activations and output gradients.
CONFIGS = {
    "C1": dict(dtype="f32", B=32, T=16, manifest=lambda: single_dense_manifest(64, 64), C=1.0,
               act_std=1.0, grad_std=0.1, data_seed=1000),
    "C2": dict(dtype="bf16", B=256, T=128, manifest=lambda: bert_manifest(12, 768, 3072), C=1.0,
               act_std=1.0, grad_std=1e-2, data_seed=1001),
    "C3": dict(dtype="bf16", B=512, T=128, manifest=lambda: bert_manifest(24, 1024, 4096, 30522, 512),
               C=1.0, act_std=1.0, grad_std=1e-2, data_seed=1002, zipf_s=1.1),
    "C4": dict(dtype="bf16", B=1024, T=128, micro_batches=64,
               manifest=lambda: bert_manifest(24, 1024, 4096, 30522, 512), C=1.0, act_std=1.0,
               grad_std=1e-2, data_seed=1003, zipf_s=1.1, sigma=0.6, noise_seed=1234, lr=1e-3,
               beta1=0.9, beta2=0.999, weight_decay=0.5),
    "C5": dict(dtype="bf16", B=128, T=512, manifest=lambda: bert_manifest(24, 1024, 4096, 30522, 512),
               C=0.5, act_std=1.0, grad_std=1e-2, data_seed=1004, zipf_s=1.1),
}
