"""The entry point that allocates nothing (dp_noise_adamw_snr_static) against the entry point it is a variant of
(dp_noise_adamw_snr), through the C ABI: two calls in a row on one stream, the second on a smaller input, so that the
second call finds the first call's partial norms in the shared static scratch array.  Both run the same kernels, so
parameters, moments, the cleared sum and the two squared norms must agree bit for bit (inside the update's tolerance
by a wide margin: rel 1e-5 on m and v, 1e-5 |theta| + 1e-3 lr on theta)."""
import numpy as np
import pytest
import torch

import dp_synth as syn

from gpu_util import DEV, f32_dev, host

pytestmark = pytest.mark.gpu


def _state(n, seed):
    th = syn.normal_f32((n,), 0.02, seed)
    m = syn.normal_f32((n,), 1e-3, seed + 1)
    v = np.abs(syn.normal_f32((n,), 1e-6, seed + 2))
    S = syn.normal_f32((n,), 30.0, seed + 3)
    return [f32_dev(x) for x in (th, m, v, S)]


def test_static_entry_point_matches_context_entry_point_twice_second_smaller():
    import paper_2108_01624_amd as pkg

    kw = dict(sigma=0.6, C=1.0, seed=1234, batch_size=4096, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-11, weight_decay=0.5)
    stream = torch.cuda.current_stream().cuda_stream
    with pkg.Context() as ctx:
        # first call: ~3.1M elements (3,073 workgroups' partial pairs), offset not a multiple of 4 (ragged head and tail);
        # second call: 70,001 elements at another offset (69 pairs: most of the first call's pairs stay behind in the scratch)
        for n, off, step, zero in ((3 * 1024 * 1024 + 517, 6, 2, True), (70_001, 4096, 3, False)):
            ref = _state(n, 9000 + step)
            got = [t.clone() for t in ref]
            snr_ref = torch.zeros(2, dtype=torch.float32, device=DEV)
            snr_got = torch.zeros(2, dtype=torch.float32, device=DEV)
            ctx.noise_adamw_snr(*ref, snr_ref, elem_offset=off, step=step, zero_sum=zero, **kw)
            pkg.dp_noise_adamw_snr_static(stream, *got, snr_got, elem_offset=off, step=step, zero_sum=zero, **kw)
            ctx.sync()
            torch.cuda.synchronize()
            for name, a, b in zip(("theta", "m", "v", "sum"), ref, got):
                np.testing.assert_array_equal(host(a).view(np.uint32), host(b).view(np.uint32), err_msg=name)
            np.testing.assert_array_equal(host(snr_ref).view(np.uint32), host(snr_got).view(np.uint32))
            assert host(snr_got)[0] > 0 and host(snr_got)[1] > 0
            assert (not host(got[3]).any()) == zero


def test_static_entry_point_rejects_what_it_cannot_hold():
    import paper_2108_01624_amd as pkg

    kw = dict(sigma=0.6, C=1.0, seed=1, step=1, batch_size=8, lr=1e-3, beta1=0.9, beta2=0.999, weight_decay=0.0)
    t = [torch.zeros(16, dtype=torch.float32, device=DEV) for _ in range(4)]
    snr = torch.zeros(2, dtype=torch.float32, device=DEV)
    with pytest.raises(pkg.DpError) as e:   # more elements than the static scratch has pairs for: refused, nothing launched
        pkg.dp_noise_adamw_snr_static(0, *t, snr, n=(1 << 30) + 1, **kw)
    assert e.value.status == -7
    with pytest.raises(pkg.DpError) as e:
        pkg.dp_noise_adamw_snr_static(0, *t, snr, **dict(kw, step=0))
    assert e.value.status == -5
    torch.cuda.synchronize()
    assert not any(host(x).any() for x in t)
