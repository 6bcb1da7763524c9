"""Algorithm 1 end to end around a small PyTorch model on synthetic data (the paper's CIFAR-10 networks
are not available): the averaged gradient that the model receives is the oracle's, bit for bit, over
chained iterations, and training with the compressed gradients converges like plain SGD."""
import numpy as np
import pytest

import oracle
import co3_inputs as inp

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def co3():
    import paper_2203_09044_amd as pkg
    return pkg


def make_problem(seed, U, batch, dim=48, classes=10):
    gen = torch.Generator().manual_seed(seed)
    centers = torch.randn(classes, dim, generator=gen) * 1.5

    def sample(t, u):
        g = torch.Generator().manual_seed(seed * 7919 + t * 131 + u)
        y = torch.randint(0, classes, (batch,), generator=g)
        x = centers[y] + torch.randn(batch, dim, generator=g)
        return x.cuda(), y.cuda()

    def model():
        torch.manual_seed(seed)
        return torch.nn.Sequential(torch.nn.Linear(dim, 300), torch.nn.ReLU(), torch.nn.Linear(300, 300),
                                   torch.nn.ReLU(), torch.nn.Linear(300, classes)).cuda()
    return sample, model


def test_average_is_the_oracles_over_chained_iterations(co3):
    from paper_2203_09044_amd.training import Co3SGD
    U, T = 3, 4
    sample, model = make_problem(5, U, 32)
    net = model()
    opt = Co3SGD(net, U, co3.Fmt(3, 1), lr=0.05)
    f = oracle.Fmt(3, 1)
    seg, n = opt.seg_off, opt.n
    errs = [np.zeros(n, np.float32) for _ in range(U)]
    loss_fn = torch.nn.functional.cross_entropy
    for t in range(T):
        before = [p.detach().clone() for p in opt.params]
        opt.local_gradients([sample(t, u) for u in range(U)], loss_fn)
        gh = opt.g[:, :n].cpu().numpy()
        opt.pipe.step(opt.g)
        assert opt.pipe.poll() == 0
        syms, A = [], []
        for u in range(U):
            a = oracle.anchor(gh[u], f, seg)
            s, errs[u] = oracle.convert_ef(gh[u], errs[u], a, 1.0, f, seg)
            syms.append(s)
            A.append(a)
            assert np.array_equal(opt.pipe.err[u, :n].cpu().numpy().view(np.uint32), errs[u].view(np.uint32))
        want = oracle.aggregate(np.stack(syms), np.stack(A), f, seg)
        assert np.array_equal(opt.pipe.avg[:n].cpu().numpy().view(np.uint32), want.view(np.uint32)), t
        opt.apply_average()
        for p, b, a0, a1 in zip(opt.params, before, seg[:-1], seg[1:]):
            upd = torch.from_numpy(want[a0:a1]).cuda().view_as(p)
            assert torch.equal(p.detach(), torch.add(b, upd, alpha=-0.05))


@pytest.mark.parametrize("E,M,bias,codes,tables", [(3, 1, "absmax", "user", "empirical"), (1, 2, "moments", "user", "empirical"),
                                                   (4, 3, "absmax", "layer", "empirical"),
                                                   (1, 2, "moments", "layer", "model"), (3, 1, "moments", "layer", "model"),
                                                   (3, 1, "absmax", "user", "lagged")])
def test_training_converges_like_plain_sgd(co3, E, M, bias, codes, tables):
    from paper_2203_09044_amd.training import Co3SGD
    U, T, lr = 4, 80, 0.1
    sample, model = make_problem(11, U, 64)
    loss_fn = torch.nn.functional.cross_entropy

    net = model()
    opt = Co3SGD(net, U, co3.Fmt(E, M), lr=lr, bias=bias, codes=codes, code_group_min=10000, tables=tables, refresh=10)
    losses = [opt.step([sample(t, u) for u in range(U)], loss_fn) for t in range(T)]
    assert opt.pipe.poll() == 0

    ref = model()                              # same initial weights, uncompressed average of the same gradients
    ref_losses = []
    for t in range(T):
        grads, tot = None, 0.0
        for u in range(U):
            ref.zero_grad(set_to_none=True)
            x, y = sample(t, u)
            l = loss_fn(ref(x), y)
            l.backward()
            tot += float(l.detach())
            gs = [p.grad.clone() for p in ref.parameters()]
            grads = gs if grads is None else [a + b for a, b in zip(grads, gs)]
        with torch.no_grad():
            for p, gsum in zip(ref.parameters(), grads):
                p.add_(gsum / U, alpha=-lr)
        ref_losses.append(tot / U)

    first, last, ref_last = np.mean(losses[:5]), np.mean(losses[-10:]), np.mean(ref_losses[-10:])
    print(f"\n[training E{E}M{M} bias={bias} codes={codes} tables={tables}] loss {first:.3f} -> {last:.3f} (plain SGD {ref_last:.3f}), "
          f"{opt.bits_per_element():.2f} payload bits per gradient element")
    assert last < 0.5 * first
    assert last < 1.35 * ref_last + 0.05
    assert opt.bits_per_element() < 1 + E + M + (0 if tables == "empirical" else 1)  # only own-count codes have that bound


def test_gradients_land_in_the_batch_rows(co3):
    """The users' gradients reach the [U][n] batch through the parameters' .grad views: every row equals the
    gradient of a plain backward pass of that user's mini-batch, tensor after tensor in parameter order."""
    from paper_2203_09044_amd.training import Co3SGD
    U = 3
    sample, model = make_problem(21, U, 16)
    net = model()
    opt = Co3SGD(net, U, co3.Fmt(3, 1), lr=0.05)
    loss_fn = torch.nn.functional.cross_entropy
    for t in range(2):                       # twice: the rows are cleared before every backward pass
        batches = [sample(t, u) for u in range(U)]
        opt.local_gradients(batches, loss_fn)
        assert all(p.grad is None for p in opt.params)
        for u, (x, y) in enumerate(batches):
            net.zero_grad(set_to_none=True)
            loss_fn(net(x), y).backward()
            want = torch.cat([p.grad.reshape(-1) for p in opt.params])
            assert torch.equal(opt.g[u, :opt.n], want), (t, u)
        net.zero_grad(set_to_none=True)


@pytest.mark.parametrize("tables,codes,bias", [("lagged", "user", "absmax"), ("model", "layer", "moments"),
                                               ("empirical", "layer", "absmax")])
def test_a_stream_that_does_not_fit_is_made_again(co3, tables, codes, bias):
    """Codes that are not built from the user's own counts of the iteration can outgrow the stream buffer.
    With a buffer far too small the wrapper must notice (device status), enlarge it and make the iteration
    again from the state before it: weights, memory, average and stream lengths equal those of a run with
    ample buffers, bit for bit."""
    from paper_2203_09044_amd.training import Co3SGD
    U, T = 3, 4
    sample, model = make_problem(31, U, 32)
    loss_fn = torch.nn.functional.cross_entropy
    runs = []
    for cap in (None, 64):
        net = model()
        opt = Co3SGD(net, U, co3.Fmt(3, 1), lr=0.05, bias=bias, codes=codes, code_group_min=10000, tables=tables,
                     refresh=2, cap_words=cap)
        for t in range(T):
            opt.step([sample(t, u) for u in range(U)], loss_fn)
        runs.append((opt, [p.detach().clone() for p in opt.params]))
    (a, pa), (b, pb) = runs
    assert a.capacity_growths == 0 and b.capacity_growths >= 1
    assert b.pipe.poll() == 0
    for x, y in zip(pa, pb):
        assert torch.equal(x, y)
    assert torch.equal(a.pipe.err.view(torch.int32), b.pipe.err.view(torch.int32))
    assert torch.equal(a.pipe.avg.view(torch.int32), b.pipe.avg.view(torch.int32))
    assert torch.equal(a.pipe.total_bits, b.pipe.total_bits)


def test_a_device_condition_other_than_capacity_raises(co3):
    from paper_2203_09044_amd.training import Co3SGD
    from paper_2203_09044_amd import binding as B
    U = 2
    sample, model = make_problem(41, U, 16)
    opt = Co3SGD(model(), U, co3.Fmt(3, 1), lr=0.05)
    before = [p.detach().clone() for p in opt.params]
    opt.pipe.status.fill_(B.EBADSTREAM)       # what a kernel would have left there
    with pytest.raises(B.Co3Error):
        opt.step([sample(0, u) for u in range(U)], torch.nn.functional.cross_entropy)
    for p, q in zip(opt.params, before):      # the average never reached the model
        assert torch.equal(p.detach(), q)
