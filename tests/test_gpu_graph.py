"""A whole step recorded into a HIP graph.

The step's entry points allocate nothing, record no memory-set nodes and never wait for the device, so a caller may
capture pass 1, pass 2 and the update of a fixed-shape micro-batch once and replay it.  Replays must give exactly what
the same calls give when issued eagerly: checked on several replays, with the program's own eager work (new inputs copied
into the captured buffers, state reset) and synchronisations between them."""
import numpy as np
import pytest
import torch

import dp_synth as syn

from gpu_util import DEV, host

pytestmark = pytest.mark.gpu

_INPUT_KEYS = ("A", "G", "X", "ids", "H", "dL")


def _load(dst_layers, src_layers):
    done = set()
    for d, s in zip(dst_layers, src_layers):
        for key in _INPUT_KEYS:
            if key in d and torch.is_tensor(d[key]) and d[key].data_ptr() not in done:
                d[key].copy_(s[key])
                done.add(d[key].data_ptr())   # tensors shared between layers (one upstream gradient) are copied once


def test_whole_step_replays_from_a_hip_graph():
    import paper_2108_01624_amd as pkg

    man = syn.bert_manifest(1, 64, 128, 97, 32, type_vocab=2)
    Bm, T, C = 8, 16, 0.05
    hp = dict(sigma=0.6, C=C, seed=77, step=1, batch_size=Bm, lr=2e-3, beta1=0.9, beta2=0.999, eps=1e-11, weight_decay=0.5)
    side = torch.cuda.Stream(device=DEV)   # default priority
    with torch.cuda.stream(side):
        with pkg.Context() as ctx:   # the context issues its work on the stream that is current when it is created
            run = pkg.StepRunner(ctx, man, Bm, device=DEV)
            mk = lambda k: syn.device_layer_inputs(man, Bm, T, dtype="bf16", act_std=1.0, grad_std=1e-2, data_seed=900 + k,
                                                   device=DEV, example_scale=syn.example_scales(Bm, 0.05, 20.0, 30 + k))
            layers = mk(0)                     # the buffers every call (and the graph) reads
            inputs = [mk(k) for k in range(3)]
            gen = torch.Generator(device=DEV)
            gen.manual_seed(5)
            theta0 = torch.randn(run.P, generator=gen, device=DEV) * 0.02

            def reset():
                run.theta.copy_(theta0)
                run.m.zero_()
                run.v.zero_()
                run.S.zero_()

            def step():
                run.pass1(layers)
                run.pass2(layers, C)
                run.update(**hp)

            refs = []
            for k in range(3):
                _load(layers, inputs[k])
                reset()
                step()
                ctx.sync()
                refs.append([host(t).copy() for t in (run.sqnorms[:Bm], run.theta, run.m, run.v, run.S)])
            assert not np.array_equal(refs[0][1], refs[1][1])   # the three inputs do differ

            _load(layers, inputs[0])
            reset()
            side.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                step()
            for k in (0, 1, 2, 1, 0):
                _load(layers, inputs[k])      # eager work between the replays ...
                reset()
                torch.cuda.synchronize()      # ... and a synchronisation
                graph.replay()
                ctx.sync()                    # also fetches the device error word: no error may be pending
                got = [host(t) for t in (run.sqnorms[:Bm], run.theta, run.m, run.v, run.S)]
                for name, g, r in zip(("sqnorms", "theta", "m", "v", "S"), got, refs[k]):
                    assert np.array_equal(g, r), (k, name, float(np.abs(g - r).max()))
            del graph
