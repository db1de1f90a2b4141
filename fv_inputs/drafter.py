"""Synthetic drafter for multi-step decoding runs.

A real drafter (the paper's SAR head) is out of scope; what a verification benchmark needs from one
is a tree some of whose paths agree with the target for a while.  Given the target's own greedy
continuation (obtained beforehand by plain one-token-at-a-time decoding), this draws, per step, how
many tokens the draft gets right along one path (geometric with per-token acceptance probability
p, capped by the tree depth and by the tokens still known), plants that many greedy tokens on one
root-to-leaf path of a seeded tree and fills every other node with random tokens.  With p around
0.75 the mean accepted length lands in the range the paper reports (about 2.8 to 4).
It holds no arithmetic of the verification method.
"""
import numpy as np

from .trees import fill_tokens, gen_tree


def draft_tree(seed: int, root_token: int, greedy_future, n_nodes: int, branching, p_accept: float, vocab: int):
    """greedy_future: the target's greedy tokens after root_token (as many as are known).
    Returns (tokens, parent, depth, n_correct)."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 7010]))
    cap = min(len(branching), len(greedy_future))
    n_correct = 0
    while n_correct < cap and rng.random() < p_accept:
        n_correct += 1
    parent, depth, planted = gen_tree(seed, n_nodes, branching, n_correct)
    good = [int(t) for t in greedy_future[:n_correct]]
    # the node after the last correct one must not continue the greedy sequence by accident,
    # or the accepted length would not be the drawn one
    avoid = None
    if n_correct < len(greedy_future):
        avoid = {i: set() for i in range(n_nodes)}
        last = int(planted[n_correct])
        for i in range(1, n_nodes):
            if int(parent[i]) == last:
                avoid[i].add(int(greedy_future[n_correct]))
    tokens = fill_tokens(seed, parent, vocab, root_token, planted, good, avoid)
    return tokens, parent, depth, n_correct
