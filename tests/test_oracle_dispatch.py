"""Pins for the oracle's Scenario-Adaptive Dispatcher (paper Sec. 3.2: a scene goes to the latency-prioritised
expert if every proposal region is near and clearly perceived, to the versatile one if some are near but unclear
or far but clear, to the accuracy-prioritised one if some are far and unclear; Sec. 4: the distance threshold is
23.5 m on KITTI and 35 m on nuScenes).

Expected values are written out by hand from those three definitions, or come from a vectorised numpy
formulation (ufunc.at + stable argsort) that shares nothing with the oracle's loops, or from invariants."""
import numpy as np
import pytest

import oracle
from paper_2507_04123_amd import gen

LPE, VEE, APE = 0, 1, 2


def _paper_thresholds():
    """The two distance thresholds the paper prints (tests/golden/, with its citation)."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "dispatcher_distance_thresholds.txt")
    vals = [float(line.split()[1]) for line in open(path) if line.strip() and not line.startswith("#")]
    assert vals == [23.5, 35.0]
    return vals


def _one_scene(rows, d, c):
    e, counts, order = oracle.dispatch(np.array(rows, np.float32).reshape(-1, 4), None, 1, d, c)
    assert counts.sum() == 1 and order.tolist() == [0] and counts[e[0]] == 1
    return int(e[0])


@pytest.mark.parametrize("d", _paper_thresholds())
def test_three_categories_as_defined(d):
    c = 0.5
    near, far = (0.5 * d, 0.0, 0.0), (0.0, 1.5 * d, 0.0)
    assert _one_scene([near + (0.9,), near + (0.6,)], d, c) == LPE                    # all close and distinct
    assert _one_scene([near + (0.9,), near + (0.2,)], d, c) == VEE                    # some near but unclear
    assert _one_scene([near + (0.9,), far + (0.8,)], d, c) == VEE                     # some far but clear
    assert _one_scene([near + (0.9,), far + (0.3,)], d, c) == APE                     # some far and unclear
    assert _one_scene([near + (0.2,), far + (0.9,), far + (0.1,)], d, c) == APE       # the hardest case decides
    assert _one_scene([], d, c) == LPE                                                 # nothing to detect
    # thresholds: "< D" is near, ">= C" is clear
    assert _one_scene([(d, 0.0, 0.0, 0.9)], d, c) == VEE                               # exactly D away: far
    assert _one_scene([(np.nextafter(np.float32(d), np.float32(0)), 0.0, 0.0, 0.5)], d, c) == LPE   # just inside, exactly C
    assert _one_scene([(3.0, 4.0, 50.0, 0.9)], 5.0 + 1e-3, c) == LPE                   # range in the ground plane: 5 m, height ignored
    assert _one_scene([(3.0, 4.0, 0.0, 0.9)], 5.0, c) == VEE
    assert _one_scene([(1.0, 1.0, 0.0, np.nan)], d, c) == VEE                          # unreadable confidence: unclear
    assert _one_scene([(np.nan, 1.0, 0.0, 0.1)], d, c) == APE                          # unreadable position: far


def _numpy_dispatch(props, scene, n_scenes, d, c):
    p = props.astype(np.float32)
    with np.errstate(invalid="ignore"):
        r2 = p[:, 0] * p[:, 0] + p[:, 1] * p[:, 1]                                     # float32 products and sum
        far = ~(r2 < np.float32(d) * np.float32(d))
        unclear = ~(p[:, 3] >= np.float32(c))
    cat = np.where(far & unclear, 2, np.where(far | unclear, 1, 0)).astype(np.int32)
    ok = (scene >= 0) & (scene < n_scenes)
    expert = np.zeros(n_scenes, np.int32)
    np.maximum.at(expert, scene[ok], cat[ok])
    return expert, np.bincount(expert, minlength=3).astype(np.int32), np.argsort(expert, kind="stable").astype(np.int32)


@pytest.mark.parametrize("n_scenes,d,c,seed", [(1, 23.5, 0.5, 1), (8, 23.5, 0.5, 2), (200, 35.0, 0.3, 3), (1000, 23.5, 0.7, 4)])
def test_matches_numpy_formulation(n_scenes, d, c, seed):
    props, scene = gen.make_proposals(n_scenes, seed, d, c)
    # a few ids outside the batch and unreadable values
    if len(props) > 10:
        scene[::97] = n_scenes + 3
        scene[5] = -1
        props[7, 3] = np.nan
    e, counts, order = oracle.dispatch(props, scene, n_scenes, d, c)
    ee, ec, eo = _numpy_dispatch(props, scene, n_scenes, d, c)
    assert np.array_equal(e, ee) and np.array_equal(counts, ec) and np.array_equal(order, eo)
    if n_scenes >= 200:
        assert counts.min() > 0.15 * n_scenes                                          # the generator covers all three classes
    # grouping: a permutation, experts non-decreasing along it, ascending scene index inside a group
    assert sorted(order.tolist()) == list(range(n_scenes))
    assert np.all(np.diff(e[order]) >= 0)
    for k in range(3):
        grp = order[counts[:k].sum():counts[:k + 1].sum()]
        assert np.all(e[grp] == k) and np.all(np.diff(grp) > 0)


def test_invariants():
    d, c, n_scenes = 23.5, 0.5, 60
    props, scene = gen.make_proposals(n_scenes, 9, d, c)
    e, counts, order = oracle.dispatch(props, scene, n_scenes, d, c)
    # the order of the proposals does not matter
    perm = gen.Stream(1, 1).permutation(len(props))
    e2, _, _ = oracle.dispatch(props[perm], scene[perm], n_scenes, d, c)
    assert np.array_equal(e, e2)
    # more proposals never lower a scene's expert; removing all of a scene's makes it LPE
    half = np.arange(len(props)) % 2 == 0
    eh, _, _ = oracle.dispatch(props[half], scene[half], n_scenes, d, c)
    assert np.all(eh <= e)
    e0, _, _ = oracle.dispatch(props[scene != 3], scene[scene != 3], n_scenes, d, c)
    assert e0[3] == LPE and np.array_equal(np.delete(e0, 3), np.delete(e, 3))
    # a larger distance threshold or a lower confidence threshold can only make scenes easier
    e_far, _, _ = oracle.dispatch(props, scene, n_scenes, 2 * d, c)
    e_lax, _, _ = oracle.dispatch(props, scene, n_scenes, d, 0.0)
    assert np.all(e_far <= e) and np.all(e_lax <= e) and np.all(e_lax <= VEE)
    # everything far and nothing clear: every non-empty scene needs the accuracy-prioritised expert
    e_all, _, _ = oracle.dispatch(props, scene, n_scenes, 0.0, 2.0)
    has = np.bincount(scene, minlength=n_scenes) > 0
    assert np.all(e_all[has] == APE) and np.all(e_all[~has] == LPE)
    with pytest.raises(RuntimeError):
        oracle.dispatch(props, scene, n_scenes, -1.0, c)


# ------------------------------------------------------------------------------------------------
# expert-grouped batching: the batch ids of the points for one expert's group
# ------------------------------------------------------------------------------------------------

def test_group_points_hand_case():
    """Five scenes, experts (1, 0, 2, 0, 1): the groups are LPE {1, 3}, VEE {0, 4}, APE {2}; a scene's slot is its
    place inside its own group, and a point gets its scene's slot only in the call for that scene's expert."""
    expert = np.array([1, 0, 2, 0, 1], np.int32)
    counts = np.array([2, 2, 1], np.int32)
    order = np.array([1, 3, 0, 4, 2], np.int32)
    scene = np.array([0, 1, 2, 3, 4, 4, 3, 7, -1, 0], np.int32)     # two ids outside the batch
    slot, gb0 = oracle.group_points(scene, len(scene), expert, order, counts, LPE)
    assert slot.tolist() == [0, 0, 0, 1, 1]
    assert gb0.tolist() == [-1, 0, -1, 1, -1, -1, 1, -1, -1, -1]
    _, gb1 = oracle.group_points(scene, len(scene), expert, order, counts, VEE)
    assert gb1.tolist() == [0, -1, -1, -1, 1, 1, -1, -1, -1, 0]
    _, gb2 = oracle.group_points(scene, len(scene), expert, order, counts, APE)
    assert gb2.tolist() == [-1, -1, 0, -1, -1, -1, -1, -1, -1, -1]
    # no scene array: every point belongs to scene 0
    _, g = oracle.group_points(None, 3, expert, order, counts, VEE)
    assert g.tolist() == [0, 0, 0]
    # an order that is not the grouping of these experts is refused
    with pytest.raises(RuntimeError):
        oracle.group_points(scene, len(scene), expert, np.array([1, 0, 3, 4, 2], np.int32), counts, LPE)


@pytest.mark.parametrize("n_scenes,seed", [(8, 3), (200, 4)])
def test_group_points_invariants_on_dispatcher_output(n_scenes, seed):
    """On the dispatcher's own output: the three calls partition the points of valid scenes; inside one group the
    slots are 0 .. count-1, ascending with the scene index; regrouping by slot reproduces `order`."""
    props, pscene = gen.make_proposals(n_scenes, seed)
    expert, counts, order = oracle.dispatch(props, pscene, n_scenes, 23.5, 0.5)
    st = gen.Stream(seed, 77)
    scene = (st.bits(5000) % np.uint64(n_scenes + 2)).astype(np.int32) - 1          # ids -1 .. n_scenes
    gbs = []
    for e in (LPE, VEE, APE):
        slot, gb = oracle.group_points(scene, len(scene), expert, order, counts, e)
        gbs.append(gb)
        mine = np.flatnonzero(expert == e)
        assert sorted(slot[mine].tolist()) == list(range(counts[e]))
        assert np.all(np.diff(slot[mine]) > 0)                                       # ascending scene index inside a group
        start = int(counts[:e].sum())
        assert np.array_equal(order[start + slot[mine]], mine)
        valid = (scene >= 0) & (scene < n_scenes)
        want = np.where(valid & (expert[np.clip(scene, 0, n_scenes - 1)] == e), slot[np.clip(scene, 0, n_scenes - 1)], -1)
        assert np.array_equal(gb, want)
    taken = np.stack(gbs) >= 0
    valid = (scene >= 0) & (scene < n_scenes)
    assert np.array_equal(taken.sum(axis=0), valid.astype(np.int64))                 # exactly one expert per valid point
