"""Next-token selection of the serving step. Oracle code: test infrastructure only.

The paper states only that temperature + top-p sampling runs on the device inside each step
(section 4.2, graph cache paragraph). The reading taken here, in this order:
  greedy when temperature == 0: the largest logit, ties to the lowest token id;
  otherwise z = logits / temperature; keep the top_k largest (ties at the boundary: lower id
  wins; top_k == 0 keeps all); softmax over the kept; order the kept by probability
  descending (ties: lower id first); keep the shortest prefix whose cumulative probability
  reaches top_p (the crossing token included); draw u in [0,1) from Philox and return the
  first token whose cumulative probability within the kept prefix exceeds u * total.
Everything is computed in fp64 from the logits given.
"""
import numpy as np

from .philox import uniform_for_token


def greedy(logits):
    logits = np.asarray(logits, dtype=np.float64)
    return int(np.argmax(logits))  # numpy returns the first (lowest-id) maximum


def candidate_order(logits):
    """Token ids by logit descending, ties by id ascending."""
    logits = np.asarray(logits, dtype=np.float64)
    return np.lexsort((np.arange(logits.size), -logits))


def sample_detail(logits, temperature, top_k, top_p, u):
    """Returns dict(token, kept (ids in order), cdf (cumulative probs of kept, unnormalised),
    total, target=u*total, margins) for a given uniform u."""
    logits = np.asarray(logits, dtype=np.float64)
    if temperature == 0.0:
        order = candidate_order(logits)
        m = float(logits[order[0]] - logits[order[1]]) if logits.size > 1 else np.inf
        return dict(token=int(order[0]), kept=order[:1], cdf=np.ones(1), total=1.0, target=0.0, logit_margin=m)
    z = logits / float(temperature)
    order = candidate_order(z)
    k = z.size if (top_k == 0 or top_k >= z.size) else int(top_k)
    cand = order[:k]
    zc = z[cand]
    p = np.exp(zc - zc[0])
    p = p / p.sum()
    cum = np.cumsum(p)
    # shortest prefix with cumulative probability >= top_p
    n_keep = int(np.searchsorted(cum, top_p, side="left")) + 1
    n_keep = min(n_keep, k)
    kept = cand[:n_keep]
    cdf = cum[:n_keep]
    total = float(cdf[-1])
    target = u * total
    idx = int(np.searchsorted(cdf, target, side="right"))
    idx = min(idx, n_keep - 1)
    return dict(token=int(kept[idx]), kept=kept, cdf=cdf, total=total, target=target,
                n_topk=k, probs=p)


def sample(logits, temperature, top_k, top_p, seed, token_index):
    """Token id for output position token_index of a request with the given sampling seed."""
    if temperature == 0.0:
        return greedy(logits)
    u = uniform_for_token(seed, token_index)
    return sample_detail(logits, temperature, top_k, top_p, u)["token"]
