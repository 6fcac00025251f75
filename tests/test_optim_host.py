"""Host-side checks of the Q-Ramping optimizer front end (no GPU: no kernel is called)."""
import pytest

torch = pytest.importorskip("torch")


def _optimizer(**kw):
    from paper_2502_20853_amd.optim import QRampingAdamW
    w = torch.nn.Parameter(torch.zeros(8, 64))
    b = torch.nn.Parameter(torch.zeros(8))
    return QRampingAdamW([w], [b], t0=3, t_update=10, **kw), w, b


def test_argument_checks():
    from paper_2502_20853_amd.optim import QRampingAdamW
    w = torch.nn.Parameter(torch.zeros(8, 64))
    for bad in (dict(t0=10, t_update=10), dict(t0=0, t_update=10), dict(n_max=0), dict(k1=0.0), dict(k2=-1)):
        with pytest.raises(ValueError):
            QRampingAdamW([w], **bad)
    with pytest.raises(ValueError):
        QRampingAdamW([torch.nn.Parameter(torch.zeros(8, 48))])               # input dimension not a multiple of 32
    with pytest.raises(ValueError):
        QRampingAdamW([w], [torch.nn.Parameter(torch.zeros(6))])              # length not a multiple of 4
    with pytest.raises(ValueError):
        QRampingAdamW([torch.nn.Parameter(torch.zeros(8, 64, dtype=torch.bfloat16))])


def test_state_dict_round_trip_keeps_integer_state():
    opt, w, b = _optimizer(lr=0.5)
    gen = torch.Generator().manual_seed(0)
    for p, q in ((w, True), (b, False)):
        st = opt._state(p, q)
        for name, t in st.items():
            if t.is_floating_point():
                t.copy_(torch.rand(t.shape, generator=gen))
            else:
                t.copy_(torch.randint(0, 200, t.shape, generator=gen).to(t.dtype))
    opt.state[w]["updates"][0, 0] = (1 << 24) + 1                             # not representable in float32
    opt.param_groups[0]["steps_done"] = 17
    saved = opt.state_dict()
    new, w2, b2 = _optimizer(lr=0.1)
    new.load_state_dict(saved)
    assert new.param_groups[0]["steps_done"] == 17 and new.param_groups[0]["lr"] == 0.5
    for p_old, p_new in ((w, w2), (b, b2)):
        assert set(new.state[p_new]) == set(opt.state[p_old])
        for name, t in opt.state[p_old].items():
            got = new.state[p_new][name]
            assert got.dtype == t.dtype and torch.equal(got, t), name
            assert got.data_ptr() != t.data_ptr()


def test_layers_get_distinct_philox_keys_by_default():
    """Two layers built with default arguments draw from different Philox keys (the upper key word
    carries the layer's construction number), and an explicit layer_id fixes the key."""
    from paper_2502_20853_amd.module import MxLinear
    a, b = MxLinear(64, 96, device="cpu"), MxLinear(64, 96, device="cpu")
    assert a.layer_id != b.layer_id and a.key_high != b.key_high
    c, d = MxLinear(64, 96, device="cpu", seed=3, layer_id=7), MxLinear(64, 96, device="cpu", seed=3, layer_id=7)
    assert c.key_high == d.key_high == ((3 << 16) | 7)
    e = MxLinear(64, 96, device="cpu", seed=3, layer_id=7, device_seed=True)
    assert int(e.seed_state.item()) & 0xFFFFFFFFFFFFFFFF == ((c.key_high << 32) - 1) & 0xFFFFFFFFFFFFFFFF
