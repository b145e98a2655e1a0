"""Paper Sec. II-C on the oracle: losing the groups with the smallest partial-output norms costs far
less output error than losing random groups, and losing the largest costs the most.  The strategies
differ only in the significance values handed to the mask builder (the norms themselves = the
predictor's training target, random values = the Random baseline, negated norms = the worst case);
the error is that of the group-sparse block against the dense one."""
import numpy as np

from oracle import ref
from tests.util import drop_strategy_case, drop_strategy_scores


def oracle_strategy_errors():
    w, K, x, Wg, Wu, WdT = drop_strategy_case()
    xn, g, u, dn = (t.float().numpy() for t in (x, Wg, Wu, WdT))
    parts = ref.group_partials(xn, g, u, dn, w.group_size)             # [T][G][d] float64
    dense = parts.sum(axis=1)
    norms = np.linalg.norm(parts, axis=2)                               # [T][G]
    pd = ref.schedule(K, [0.0])                                         # one lossless device
    errs = {}
    for name, sc in drop_strategy_scores(w, norms).items():
        mask = ref.build_group_mask(sc, K, pd, 1, None)["mask"]
        assert (mask.sum(axis=1) == K).all()
        y = ref.group_sparse_ffn(xn, g, u, dn, w.group_size, mask)
        # the sparse block is the dense one minus the partial results that were left out
        lost = (parts * (1 - mask)[:, :, None]).sum(axis=1)
        np.testing.assert_allclose(y, dense - lost, rtol=0, atol=1e-12 * np.abs(dense).max())
        errs[name] = float((np.linalg.norm(y - dense, axis=1) / np.linalg.norm(dense, axis=1)).mean())
    return errs, norms


def test_low_norm_ordering_loses_less_than_random_and_random_less_than_high_norm():
    errs, norms = oracle_strategy_errors()
    assert errs["low_norm"] < 0.6 * errs["random"] < errs["high_norm"], errs
    # the synthetic groups really are imbalanced: the largest norm of a token is several times its median
    assert (norms.max(axis=1) > 4 * np.median(norms, axis=1)).all()


def test_keeping_the_top_k_norms_is_the_best_k_subset_for_nearly_orthogonal_partials():
    # with random weights the partial results are nearly orthogonal, so the squared error of leaving a
    # set out is close to the sum of its squared norms: no random K-subset may beat the top-K one by
    # more than the cross terms allow
    w, K, x, Wg, Wu, WdT = drop_strategy_case()
    xn, g, u, dn = (t.float().numpy() for t in (x, Wg, Wu, WdT))
    parts = ref.group_partials(xn, g, u, dn, w.group_size)
    dense = parts.sum(axis=1)
    norms = np.linalg.norm(parts, axis=2)
    rng = np.random.default_rng(5)
    G = w.n_groups
    for t in range(w.T):
        top = np.argsort(-norms[t], kind="stable")[:K]
        e_top = np.linalg.norm(dense[t] - parts[t, top].sum(axis=0))
        for _ in range(200):
            sub = rng.choice(G, size=K, replace=False)
            e_sub = np.linalg.norm(dense[t] - parts[t, sub].sum(axis=0))
            assert e_top <= e_sub * 1.05
