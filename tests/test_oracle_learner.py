"""Pins of the learner oracle (oracle/msrl_learn_ref.c): CPU only.

The update rule is the PPO clipped surrogate the oracle's header states.  It is pinned to things
other than itself: an automatic-differentiation library evaluating the same objective (loss and
every gradient; both action distributions; rows in every clip regime; the bf16 straight-through
rule), central finite differences of the loss, closed forms at all-zero parameters, the exact zero
of the policy gradient when every row is clipped, and Adam's one- and two-step closed forms.
"""
import numpy as np
import pytest
import torch

from oracle import ref

LN2PI_HALF = 0.91893853320467274178


def split_params(p, i, h, o, layers=2):
    s, out = 0, []
    shapes = [(i, h), (h,)] + [(h, h), (h,)] * (layers - 1) + [(h, o), (o,)]
    for shape in shapes:
        n = int(np.prod(shape))
        out.append(p[s:s + n].reshape(shape))
        s += n
    return out, s


def bf16_ste(x):
    """Round to bfloat16 (nearest even) in the value, identity in the derivative."""
    r = x.detach().to(torch.float32).to(torch.bfloat16).to(torch.float64)
    return x + (r - x).detach()


def to_bf16(t):
    return t.to(torch.float32).to(torch.bfloat16).to(torch.float64)


class RoundGradient(torch.autograd.Function):
    """Identity; the gradient that flows back through it is rounded to bfloat16."""

    @staticmethod
    def forward(ctx, x):
        return x.clone()

    @staticmethod
    def backward(ctx, g):
        return to_bf16(g)


class TanhRoundedBackward(torch.autograd.Function):
    """tanh whose derivative is taken at the bfloat16-rounded output, the result rounded to bfloat16."""

    @staticmethod
    def forward(ctx, z):
        a = torch.tanh(z)
        ctx.save_for_backward(to_bf16(a))
        return a

    @staticmethod
    def backward(ctx, g):
        (ar,) = ctx.saved_tensors
        return to_bf16(g * (1.0 - ar * ar))


def torch_objective(pol, cfg, params, obs, actions, logp_old, adv, ret, backward_rounding=True):
    """The objective written with library tensor ops; gradients come from autograd.  In bf16 mode the
    roundings of the forward pass are straight-through; with backward_rounding the gradient is also
    rounded to bfloat16 at the network output and at every pre-activation, and tanh' uses the rounded
    activation (the oracle's reading of a bf16 backward pass)."""
    P = torch.tensor(params, dtype=torch.float64, requires_grad=True)
    rnd = bf16_ste if pol.bf16 else (lambda t: t)
    rb = pol.bf16 and backward_rounding
    act = TanhRoundedBackward.apply if rb else torch.tanh
    outg = RoundGradient.apply if rb else (lambda t: t)

    def net(p, out, x, width):
        parts, used = split_params(p, width, pol.hidden, out, pol.hidden_layers)
        h = torch.tensor(x, dtype=torch.float64)
        for l in range(pol.hidden_layers):
            h = act(rnd(h) @ rnd(parts[2 * l]) + parts[2 * l + 1])
        return outg(rnd(h) @ rnd(parts[-2]) + parts[-1]), used

    obs = np.asarray(obs, dtype=np.float64)
    y, used = net(P, pol.out_dim, obs, pol.in_dim)
    G = pol.value_in_dim // pol.in_dim       # > 1: centralised critic on groups of G consecutive rows
    v, _ = net(P[used:], 1, obs.reshape(-1, pol.value_in_dim), pol.value_in_dim)
    A = torch.tensor(adv, dtype=torch.float64)
    if pol.dist == ref.CATEGORICAL:
        lsm = torch.log_softmax(y, dim=1)
        logp = lsm.gather(1, torch.tensor(actions, dtype=torch.int64)[:, None])[:, 0]
        ent = -(lsm.exp() * lsm).sum(1)
    else:
        K = pol.out_dim // 2
        dist = torch.distributions.Normal(y[:, :K], y[:, K:].exp())
        logp = dist.log_prob(torch.tensor(actions, dtype=torch.float64)).sum(1)
        ent = dist.entropy().sum(1)
    rho = (logp - torch.tensor(logp_old, dtype=torch.float64)).exp()
    surr = torch.minimum(rho * A, rho.clamp(1 - cfg.clip, 1 + cfg.clip) * A)
    target = torch.tensor(np.asarray(ret, dtype=np.float64)[::G].copy(), dtype=torch.float64)
    loss = (-surr - cfg.ent_coef * ent).mean() + cfg.vf_coef * ((v[:, 0] - target) ** 2).mean()
    loss.backward()
    return float(loss.detach()), P.grad.numpy(), float(ent.mean().detach())


def make_case(dist, bf16, seed, R=41, i=6, h=8, K=3, layers=2, group=1):
    rng = np.random.default_rng(seed)
    o = 5 if dist == ref.CATEGORICAL else 2 * K
    pol = ref.Policy(i, h, o, bf16=bf16, dist=dist, hidden_layers=layers, value_in_dim=group * i if group > 1 else 0)
    params = rng.normal(0, 0.6, pol.param_count)
    obs = rng.normal(0, 1, (R, i))
    if dist == ref.CATEGORICAL:
        actions = rng.integers(0, o, R).astype(np.int32)
    else:
        actions = rng.normal(0, 1, (R, K))
    adv = rng.normal(0, 1, R)
    ret = rng.normal(0, 1, R)
    # old log-probabilities that put the ratios below, inside and above the clip range
    cfg0 = ref.ppo_cfg()
    _, _, st = ref.ppo_loss(pol, cfg0, params, obs, actions, np.zeros(R), adv, ret, want_grad=False)
    logp_new = np.zeros(R)
    # (a single row is no whole group: the probe uses the policy network with a per-row value net of zeros)
    own = ref.Policy(i, h, o, bf16=bf16, dist=dist, hidden_layers=layers)
    p_own = np.concatenate([params[:pol.policy_param_count], np.zeros(own.param_count - own.policy_param_count)])
    for n in range(R):   # logp of each row from a single-row call with logp_old = 0: stats[4] = -logp
        _, _, s1 = ref.ppo_loss(own, cfg0, p_own, obs[n:n + 1], actions[n:n + 1], np.zeros(1), adv[n:n + 1],
                                ret[n:n + 1], want_grad=False)
        logp_new[n] = -s1[4]
    logp_old = logp_new - rng.choice([-0.5, -0.1, 0.0, 0.1, 0.5], R)
    return pol, params, obs, actions, logp_old, adv, ret


@pytest.mark.parametrize("dist", [ref.CATEGORICAL, ref.DIAG_GAUSSIAN])
@pytest.mark.parametrize("bf16", [False, True])
def test_loss_and_gradient_against_autograd(dist, bf16):
    pol, params, obs, actions, logp_old, adv, ret = make_case(dist, bf16, 3 + dist)
    cfg = ref.ppo_cfg(clip=0.2, vf_coef=0.7, ent_coef=0.03)
    loss, grad, stats = ref.ppo_loss(pol, cfg, params, obs, actions, logp_old, adv, ret)
    t_loss, t_grad, t_ent = torch_objective(pol, cfg, params, obs, actions, logp_old, adv, ret)
    assert 0.1 < stats[3] < 0.9            # both branches of the min occur
    np.testing.assert_allclose(loss, t_loss, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(stats[2], t_ent, rtol=1e-11)
    np.testing.assert_allclose(grad, t_grad, rtol=1e-9, atol=1e-12)


@pytest.mark.parametrize("dist", [ref.CATEGORICAL, ref.DIAG_GAUSSIAN])
@pytest.mark.parametrize("layers", [2, 4])
def test_bf16_backward_roundings_are_small_and_where_stated(dist, layers):
    # The bf16 backward pass rounds dL/dy and every dL/d(pre-activation) to bfloat16 and takes tanh' at
    # the rounded activation.  (a) That gradient stays within the bf16 tolerance (2e-2) of the one without those
    # roundings (per network, in the Euclidean norm); (b) it is not the same gradient (the
    # roundings are really there); (c) with operands that bf16 holds exactly the two coincide.
    pol, params, obs, actions, logp_old, adv, ret = make_case(dist, True, 60 + dist + layers, R=64, layers=layers)
    cfg = ref.ppo_cfg(clip=0.2, vf_coef=0.7, ent_coef=0.03)
    _, grad, _ = ref.ppo_loss(pol, cfg, params, obs, actions, logp_old, adv, ret)
    _, g_plain, _ = torch_objective(pol, cfg, params, obs, actions, logp_old, adv, ret, backward_rounding=False)
    n_pi = pol.policy_param_count
    for sl in (slice(0, n_pi), slice(n_pi, None)):       # per network, in the Euclidean norm
        assert np.linalg.norm(grad[sl] - g_plain[sl]) <= 2e-2 * np.linalg.norm(g_plain[sl])
    assert np.abs(grad - g_plain).max() > 0
    # every rounding point of the backward pass is exact: no hidden layer (tanh never runs), and
    # dL/dy a dyadic number -- one row, value net only: dv = c_v 2 (b - ret) with all weights zero
    lin = ref.Policy(4, 8, 5, bf16=True, hidden_layers=1)
    p0 = np.zeros(lin.param_count)
    p0[-1] = 0.75
    x = np.array([[0.5, -0.25, 1.0, 2.0]])
    _, g1, _ = ref.ppo_loss(lin, ref.ppo_cfg(vf_coef=0.5, ent_coef=0.0), p0, x, np.array([1], np.int32),
                            np.array([-np.log(5.0)]), np.zeros(1), np.array([0.25]))
    assert g1[-1] == 0.5 * 2 * 0.5            # output bias of the value net: dv = 0.5, representable
    _, g2, _ = torch_objective(lin, ref.ppo_cfg(vf_coef=0.5, ent_coef=0.0), p0, x, np.array([1], np.int32),
                               np.array([-np.log(5.0)]), np.zeros(1), np.array([0.25]), backward_rounding=False)
    np.testing.assert_allclose(g1[lin.policy_param_count:], g2[lin.policy_param_count:], rtol=1e-15, atol=0)


@pytest.mark.parametrize("dist,bf16,group", [(ref.CATEGORICAL, False, 3), (ref.CATEGORICAL, True, 4),
                                             (ref.DIAG_GAUSSIAN, False, 2)])
def test_centralised_critic_against_autograd(dist, bf16, group):
    # the value network on groups of `group` consecutive rows (the agents of an env), one target per group
    pol, params, obs, actions, logp_old, adv, ret = make_case(dist, bf16, 30 + group, R=12 * group, group=group)
    assert pol.value_in_dim == group * pol.in_dim
    cfg = ref.ppo_cfg(clip=0.2, vf_coef=0.7, ent_coef=0.03)
    loss, grad, stats = ref.ppo_loss(pol, cfg, params, obs, actions, logp_old, adv, ret)
    t_loss, t_grad, t_ent = torch_objective(pol, cfg, params, obs, actions, logp_old, adv, ret)
    np.testing.assert_allclose(loss, t_loss, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(grad, t_grad, rtol=1e-9, atol=1e-12)
    assert np.abs(grad[pol.policy_param_count:]).min() >= 0 and np.abs(grad[pol.policy_param_count:]).max() > 1e-4
    # targets other than the group's first row are not used
    ret2 = ret.copy()
    ret2[np.arange(ret.size) % group != 0] += 5.0
    loss2, grad2, _ = ref.ppo_loss(pol, cfg, params, obs, actions, logp_old, adv, ret2)
    assert loss2 == loss and (grad2 == grad).all()


def test_centralised_critic_reduces_to_the_per_row_value_net():
    # width in_dim (a group of one row) is the per-row learner; and a critic that looks at the group's first
    # row only has the value loss and value-net gradient of the per-row learner on those rows
    group = 3
    pol, params, obs, actions, logp_old, adv, ret = make_case(ref.CATEGORICAL, False, 41, R=30, group=group)
    cfg = ref.ppo_cfg(vf_coef=0.9)
    i, h = pol.in_dim, pol.hidden
    own = ref.Policy(i, h, pol.out_dim)
    same = ref.Policy(i, h, pol.out_dim, value_in_dim=i)
    n_pi = pol.policy_param_count
    p_own = np.concatenate([params[:n_pi], params[n_pi:n_pi + i * h], params[n_pi + group * i * h:]])
    a = ref.ppo_loss(own, cfg, p_own, obs, actions, logp_old, adv, ret)
    b = ref.ppo_loss(same, cfg, p_own, obs, actions, logp_old, adv, ret)
    assert a[0] == b[0] and (a[1] == b[1]).all()
    pc = params.copy()
    pc[n_pi + i * h:n_pi + group * i * h] = 0          # W1 rows of the other agents
    _, g_c, st_c = ref.ppo_loss(pol, cfg, pc, obs, actions, logp_old, adv, ret)
    first = slice(0, None, group)
    _, g_o, st_o = ref.ppo_loss(own, cfg, p_own, obs[first], actions[first], logp_old[first], adv[first], ret[first])
    np.testing.assert_allclose(st_c[1], st_o[1], rtol=1e-13)
    np.testing.assert_allclose(g_c[n_pi:n_pi + i * h], g_o[n_pi:n_pi + i * h], rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(g_c[n_pi + group * i * h:], g_o[n_pi + i * h:], rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("layers", [1, 3, 5])
@pytest.mark.parametrize("dist,bf16", [(ref.CATEGORICAL, False), (ref.CATEGORICAL, True), (ref.DIAG_GAUSSIAN, False)])
def test_deeper_networks_against_autograd(layers, dist, bf16):
    pol, params, obs, actions, logp_old, adv, ret = make_case(dist, bf16, 40 + layers + dist, R=23, layers=layers)
    cfg = ref.ppo_cfg(clip=0.2, vf_coef=0.7, ent_coef=0.03)
    loss, grad, stats = ref.ppo_loss(pol, cfg, params, obs, actions, logp_old, adv, ret)
    t_loss, t_grad, t_ent = torch_objective(pol, cfg, params, obs, actions, logp_old, adv, ret)
    np.testing.assert_allclose(loss, t_loss, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(stats[2], t_ent, rtol=1e-11)
    np.testing.assert_allclose(grad, t_grad, rtol=1e-9, atol=1e-12)
    assert np.abs(grad).min() >= 0 and np.count_nonzero(grad) > 0.9 * grad.size


def test_deeper_network_against_finite_differences():
    pol, params, obs, actions, logp_old, adv, ret = make_case(ref.CATEGORICAL, False, 77, R=13, layers=4)
    cfg = ref.ppo_cfg(ent_coef=0.02)
    _, grad, _ = ref.ppo_loss(pol, cfg, params, obs, actions, logp_old, adv, ret)
    rng = np.random.default_rng(0)
    for j in rng.choice(params.size, 40, replace=False):
        e = np.zeros_like(params)
        e[j] = 1e-6
        lp, _, _ = ref.ppo_loss(pol, cfg, params + e, obs, actions, logp_old, adv, ret, want_grad=False)
        lm, _, _ = ref.ppo_loss(pol, cfg, params - e, obs, actions, logp_old, adv, ret, want_grad=False)
        np.testing.assert_allclose(grad[j], (lp - lm) / 2e-6, rtol=2e-5, atol=1e-8)


@pytest.mark.parametrize("dist", [ref.CATEGORICAL, ref.DIAG_GAUSSIAN])
def test_gradient_against_finite_differences(dist):
    pol, params, obs, actions, logp_old, adv, ret = make_case(dist, False, 11 + dist, R=17)
    cfg = ref.ppo_cfg(ent_coef=0.02)
    _, grad, _ = ref.ppo_loss(pol, cfg, params, obs, actions, logp_old, adv, ret)
    rng = np.random.default_rng(0)
    for j in rng.choice(params.size, 40, replace=False):
        e = np.zeros_like(params)
        e[j] = 1e-6
        lp, _, _ = ref.ppo_loss(pol, cfg, params + e, obs, actions, logp_old, adv, ret, want_grad=False)
        lm, _, _ = ref.ppo_loss(pol, cfg, params - e, obs, actions, logp_old, adv, ret, want_grad=False)
        np.testing.assert_allclose(grad[j], (lp - lm) / 2e-6, rtol=2e-5, atol=1e-8)


def test_closed_forms_at_zero_parameters():
    rng = np.random.default_rng(1)
    R = 29
    adv, ret = rng.normal(0, 1, R), rng.normal(0, 1, R)
    cfg = ref.ppo_cfg(vf_coef=0.5, ent_coef=0.01)
    # categorical: uniform over 5 actions, ratio 1 when the old policy was uniform too
    pol = ref.Policy(4, 8, 5)
    loss, grad, st = ref.ppo_loss(pol, cfg, np.zeros(pol.param_count), rng.normal(0, 1, (R, 4)),
                                  rng.integers(0, 5, R), np.full(R, -np.log(5.0)), adv, ret)
    np.testing.assert_allclose(st[:3], [-adv.mean(), (ret ** 2).mean(), np.log(5.0)], rtol=1e-12)
    np.testing.assert_allclose(loss, -adv.mean() + 0.5 * (ret ** 2).mean() - 0.01 * np.log(5.0), rtol=1e-12)
    # only the output biases see a gradient when every weight is zero; the value bias gets c_v 2 mean(0 - ret)
    used = ref.net_param_count(4, 8, 5)
    np.testing.assert_allclose(grad[-1], 0.5 * 2.0 * (-ret).mean(), rtol=1e-12)
    assert np.count_nonzero(grad[:used - 5]) == 0
    # Gaussian: mean 0, unit standard deviation
    K = 3
    polg = ref.Policy(4, 8, 2 * K, dist=ref.DIAG_GAUSSIAN)
    a = rng.normal(0, 1, (R, K))
    lp_old = -0.5 * (a ** 2).sum(1) - K * LN2PI_HALF
    loss, _, st = ref.ppo_loss(polg, cfg, np.zeros(polg.param_count), rng.normal(0, 1, (R, 4)), a, lp_old, adv, ret)
    np.testing.assert_allclose(st[:3], [-adv.mean(), (ret ** 2).mean(), K * (LN2PI_HALF + 0.5)], rtol=1e-12)
    np.testing.assert_allclose(st[4], 0.0, atol=1e-14)


def test_clipped_rows_give_no_policy_gradient():
    pol, params, obs, actions, _, adv, ret = make_case(ref.CATEGORICAL, False, 5)
    cfg = ref.ppo_cfg(ent_coef=0.0)
    # make every ratio exp(0.5) > 1 + clip and every advantage positive: the min is the clipped, flat branch
    logp_new = np.array([-ref.ppo_loss(pol, cfg, params, obs[n:n + 1], actions[n:n + 1], np.zeros(1), np.ones(1),
                                       ret[n:n + 1], want_grad=False)[2][4] for n in range(adv.size)])
    _, grad, st = ref.ppo_loss(pol, cfg, params, obs, actions, logp_new - 0.5, np.abs(adv) + 0.1, ret)
    used = ref.net_param_count(pol.in_dim, pol.hidden, pol.out_dim)
    assert st[3] == 1.0
    assert np.count_nonzero(grad[:used]) == 0 and np.count_nonzero(grad[used:]) > 0
    # and with negative advantages the same ratios are not clipped
    _, grad, st = ref.ppo_loss(pol, cfg, params, obs, actions, logp_new - 0.5, -np.abs(adv) - 0.1, ret)
    assert st[3] == 0.0 and np.count_nonzero(grad[:used]) > 0


def test_adam_closed_forms_and_update_loop():
    cfg = ref.ppo_cfg(lr=1e-2, beta1=0.9, beta2=0.999, adam_eps=1e-8)
    rng = np.random.default_rng(2)
    g = rng.normal(0, 1, 50)
    p0 = rng.normal(0, 1, 50)
    p, m, v = p0.copy(), np.zeros(50), np.zeros(50)
    ref.adam_step(cfg, p, m, v, g, 1)
    step = -1e-2 * g / (np.abs(g) + 1e-8)          # bias-corrected moments after one step: g and g^2
    np.testing.assert_allclose(p - p0, step, rtol=1e-12)
    ref.adam_step(cfg, p, m, v, g, 2)              # same gradient again: same corrected moments, same step
    np.testing.assert_allclose(p - p0, 2 * step, rtol=1e-12)
    np.testing.assert_allclose(m, (1 - 0.9 ** 2) * g, rtol=1e-12)
    np.testing.assert_allclose(v, (1 - 0.999 ** 2) * g * g, rtol=1e-12)
    # the update loop = the same steps taken by hand, minibatch by minibatch, epoch by epoch
    pol, params, obs, actions, logp_old, adv, ret = make_case(ref.CATEGORICAL, False, 9, R=30)
    pa, ma, va = params.copy(), np.zeros_like(params), np.zeros_like(params)
    mean_loss, k = ref.ppo_update(pol, cfg, pa, ma, va, 0, 2, 3, obs, actions, logp_old, adv, ret)
    pb, mb, vb, kk, losses = params.copy(), np.zeros_like(params), np.zeros_like(params), 0, []
    for it in range(2):
        for b in range(3):
            sl = slice(10 * b, 10 * b + 10)
            l, gr, _ = ref.ppo_loss(pol, cfg, pb, obs[sl], actions[sl], logp_old[sl], adv[sl], ret[sl])
            kk += 1
            ref.adam_step(cfg, pb, mb, vb, gr, kk)
            losses.append(l)
    assert k == 6
    np.testing.assert_allclose(pa, pb, rtol=1e-13)
    np.testing.assert_allclose(mean_loss, np.mean(losses), rtol=1e-13)
    assert np.mean(losses[3:]) < np.mean(losses[:3])    # the second pass starts from improved parameters
